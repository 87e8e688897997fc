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
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = wave_id();
  const int b0 = blockIdx.y * BC;
  const int nb = min(BC, a.B - b0);
  const T* h = static_cast<const T*>(a.h);
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
  block_sums<BC>(psum, s_red, mean);
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
#pragma unroll
  for (int bc = 0; bc < BC; ++bc) {
    const float s = wave_total(acc[bc]);
    if (lane == 0 && bc < nb)
      a.z[static_cast<int64_t>(b0 + bc) * a.hidden + r] = gelu_erf(s + to_float(static_cast<const T*>(a.b1)[r]));
  }
}

template <typename T, int BC>
__global__ __launch_bounds__(kPredThreads) void output_kernel(PredictArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int kStep = kWave * EPL;
  extern __shared__ float s_z[];  // [BC][staged_len(hidden)]
  const int h_pad = staged_len<EPL>(a.hidden);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = wave_id();
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

// ---- batched form on the matrix cores (bf16, 8 sequences or more).  With a batch the two
// layers are [B x E] x [E x hidden] and [B x hidden] x [hidden x out] products; the FMA kernels
// above spend one instruction per (weight, sequence) pair, the MFMA form one
// v_mfma_f32_16x16x16_bf16 per 16 x 16 outputs and 16 inputs.  The batch is the M side (16 rows
// per tile, rows past B are computed on a clamped row and dropped), 16 output rows of the weight
// matrix the N side.  A lane loads 8 consecutive inputs of its weight row (one 128-bit load) and
// of its sequence's activations (fp32, two 128-bit loads); the two halves feed two MFMAs whose
// 16 inputs are {8q .. 8q+3} and {8q+4 .. 8q+7} of each quarter q of a 32-input step -- any
// assignment of inputs to the k slots is right as long as both operands use the same one.
// The fp32 activations enter as a sum of two bf16 numbers (the value rounded to bf16, and the
// rounded remainder): two MFMAs per weight fragment, 2^-17 relative error per product instead
// of 2^-9, so the fp32-accumulation contract of the FMA path is kept.
typedef short mfma_bf16x4 __attribute__((ext_vector_type(4)));
typedef float mfma_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t pred_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaK = 32;            // inputs per step of a wave
constexpr int kHidMfmaWaves = 16;     // waves of a hidden-layer workgroup: they split the inputs
constexpr int kOutMfmaWaves = 4;      // waves of an output-layer workgroup: one 16-row tile each

// Operands of one 32-input step for M tile rows `x` (fp32 activations of this lane's sequence,
// 8 consecutive inputs) and weight row `w` (8 consecutive bf16): acc += x . w over the step.
typedef __bf16 pred_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pred_f32x2 __attribute__((ext_vector_type(2)));

__device__ inline void mfma_step(const float (&x)[8], const pred_u32x4& w, mfma_f32x4& acc) {
  // pairs of activations -> packed bf16 pairs (round to nearest even; one conversion instruction
  // per pair on this chip), the remainders x - hi (exact in fp32) the same way
  uint32_t hi[4], lo[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const pred_bf16x2 h = __builtin_convertvector(pred_f32x2{x[2 * i], x[2 * i + 1]}, pred_bf16x2);
    __builtin_memcpy(&hi[i], &h, 4);
    const float r0 = x[2 * i] - __uint_as_float(hi[i] << 16);
    const float r1 = x[2 * i + 1] - __uint_as_float(hi[i] & 0xFFFF0000u);
    const pred_bf16x2 l = __builtin_convertvector(pred_f32x2{r0, r1}, pred_bf16x2);
    __builtin_memcpy(&lo[i], &l, 4);
  }
  auto frag = [](uint32_t p0, uint32_t p1) {
    mfma_bf16x4 r;
    __builtin_memcpy(&r, &p0, 4);
    __builtin_memcpy(reinterpret_cast<char*>(&r) + 4, &p1, 4);
    return r;
  };
  mfma_bf16x4 w0, w1;
  __builtin_memcpy(&w0, &w, 8);
  __builtin_memcpy(&w1, reinterpret_cast<const char*>(&w) + 8, 8);
  acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag(hi[0], hi[1]), w0, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag(lo[0], lo[1]), w0, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag(hi[2], hi[3]), w1, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(frag(lo[2], lo[3]), w1, acc, 0, 0, 0);
}

// The steps k_first, k_first + stride, ... < K of a wave.  The loads of 8/MT steps (weights and
// activations) are issued before the first of them is used: one memory round trip per chunk
// instead of one per step.  A step past the end reads a clamped address and is skipped.
template <int MT>
__device__ inline void mfma_walk(const bf16_t* wrow, const float* const (&xrow)[MT], int k_first, int stride, int K,
                                 mfma_f32x4 (&acc)[MT]) {
  constexpr int CH = 8 / MT;
  for (int kc = k_first; kc < K; kc += CH * stride) {
    pred_u32x4 w[CH];
    float4 xa[CH][MT], xb[CH][MT];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int k = kc + c * stride;
      const int ks = k < K ? k : K - kMfmaK;
      w[c] = *reinterpret_cast<const pred_u32x4*>(wrow + ks);
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        xa[c][m] = *reinterpret_cast<const float4*>(xrow[m] + ks);
        xb[c][m] = *reinterpret_cast<const float4*>(xrow[m] + ks + 4);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      if (kc + c * stride < K) {  // (the same for every lane of the wave)
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const float x[8] = {xa[c][m].x, xa[c][m].y, xa[c][m].z, xa[c][m].w,
                              xb[c][m].x, xb[c][m].y, xb[c][m].z, xb[c][m].w};
          mfma_step(x, w[c], acc[m]);
        }
      }
    }
  }
}

// z[b][n] = gelu(W1[n] . xln[b] + b1[n]) for 16 hidden units n and MT*16 sequences per
// workgroup; the 16 waves take every 16th step of the E inputs and their partial tiles are
// summed through LDS (in wave order: reproducible).
template <int MT>
__global__ __launch_bounds__(kHidMfmaWaves * kWave) void hidden_mfma_kernel(PredictArgs a) {
  __shared__ float s_red[kHidMfmaWaves][MT][256];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = wave_id();
  const int r = lane % 16, q = lane / 16;
  const int n0 = blockIdx.x * 16, b0 = blockIdx.y * (16 * MT);
  const bf16_t* wrow = static_cast<const bf16_t*>(a.W1) + static_cast<int64_t>(n0 + r) * a.E + q * 8;
  const float* xrow[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int b = b0 + m * 16 + r;
    xrow[m] = a.xln + static_cast<int64_t>(b < a.B ? b : a.B - 1) * a.E + q * 8;
  }
  mfma_f32x4 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = mfma_f32x4{0.f, 0.f, 0.f, 0.f};
  mfma_walk<MT>(wrow, xrow, wave * kMfmaK, kHidMfmaWaves * kMfmaK, a.E, acc);
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 4; ++v) s_red[wave][m][lane * 4 + v] = acc[m][v];
  __syncthreads();
  // element e = lane*4 + v of a tile is (sequence 4*(lane/16) + v, unit lane%16)
  for (int t = tid; t < MT * 256; t += kHidMfmaWaves * kWave) {
    const int m = t / 256, e = t % 256;
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kHidMfmaWaves; ++w) sum += s_red[w][m][e];
    const int l = e / 4, v = e % 4;
    const int b = b0 + m * 16 + 4 * (l / 16) + v, n = n0 + l % 16;
    if (b < a.B) a.z[static_cast<int64_t>(b) * a.hidden + n] = gelu_erf(sum + to_float(static_cast<const bf16_t*>(a.b1)[n]));
  }
}

// y[b][o] = W2[o] . z[b] + b2[o] for 16 output rows o per wave and MT*16 sequences, rounded to
// bf16 and scattered to q_imp[slot][b][head][j].
template <int MT>
__global__ __launch_bounds__(kOutMfmaWaves * kWave) void output_mfma_kernel(PredictArgs a) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = wave_id();
  const int r = lane % 16, q = lane / 16;
  const int n_out = a.G * a.Hq * a.Dimp;
  const int n0 = (blockIdx.x * kOutMfmaWaves + wave) * 16, b0 = blockIdx.y * (16 * MT);
  if (n0 >= n_out) return;
  const bf16_t* wrow = static_cast<const bf16_t*>(a.W2) + static_cast<int64_t>(n0 + r) * a.hidden + q * 8;
  const float* xrow[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int b = b0 + m * 16 + r;
    xrow[m] = a.z + static_cast<int64_t>(b < a.B ? b : a.B - 1) * a.hidden + q * 8;
  }
  mfma_f32x4 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = mfma_f32x4{0.f, 0.f, 0.f, 0.f};
  mfma_walk<MT>(wrow, xrow, 0, kMfmaK, a.hidden, acc);
  const int o = n0 + r;  // this lane's output row: (slot, head, j), slot outermost
  const int per_slot = a.Hq * a.Dimp;
  const int slot = o / per_slot, rest = o % per_slot;
  const float bias = to_float(static_cast<const bf16_t*>(a.b2)[o]);
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int b = b0 + m * 16 + 4 * q + v;
      if (b < a.B)
        store_elt(static_cast<bf16_t*>(a.q_imp) + (static_cast<int64_t>(slot) * a.B + b) * per_slot + rest,
                  acc[m][v] + bias);
    }
}

// bf16 batches of 8 or more whose sizes fit the tiles
bool mfma_form_serves(const PredictArgs& a) {
  return a.B >= 8 && a.E % kMfmaK == 0 && a.hidden % kMfmaK == 0 && a.hidden % 16 == 0 &&
         (a.G * a.Hq * a.Dimp) % 16 == 0 && a.xln != nullptr && (reinterpret_cast<uintptr_t>(a.z) & 15u) == 0;
}

tb_status launch_mfma(const PredictArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((ln_kernel<bf16_t>), dim3(a.B), dim3(kPredThreads), 0, st, a);
  if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
  const int n_out = a.G * a.Hq * a.Dimp;
  const bool two = a.B > 16;  // 32 sequences per workgroup read every weight once for two M tiles
  const unsigned groups = static_cast<unsigned>((a.B + (two ? 32 : 16) - 1) / (two ? 32 : 16));
  const dim3 hgrid(static_cast<unsigned>(a.hidden / 16), groups), hblock(kHidMfmaWaves * kWave);
  const dim3 ogrid(static_cast<unsigned>((n_out / 16 + kOutMfmaWaves - 1) / kOutMfmaWaves), groups),
      oblock(kOutMfmaWaves * kWave);
  if (two) {
    hipLaunchKernelGGL((hidden_mfma_kernel<2>), hgrid, hblock, 0, st, a);
    if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
    hipLaunchKernelGGL((output_mfma_kernel<2>), ogrid, oblock, 0, st, a);
  } else {
    hipLaunchKernelGGL((hidden_mfma_kernel<1>), hgrid, hblock, 0, st, a);
    if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
    hipLaunchKernelGGL((output_mfma_kernel<1>), ogrid, oblock, 0, st, a);
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
  if (L.dtype == TB_BF16 && mfma_form_serves(a)) return launch_mfma(a, st);
  return L.dtype == TB_F32 ? launch_t<float>(a, st) : launch_t<bf16_t>(a, st);
}

}  // namespace tb
