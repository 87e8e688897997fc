// Importance scoring: scores[b,h,n] = scale * <q_imp[b,h,:], K_imp[b,h/g,n,:]>.
//
// Bandwidth-bound stream over the projected-key cache.  A projected row is Dimp*sizeof(T)
// bytes (64 B for the Llama-shaped configs); LPR = row_bytes/16 adjacent lanes each take one
// 128-bit load of a row, so a wave instruction reads 1 KiB of consecutive memory.  Every
// loaded row is used for all g query heads of its KV head (the cache is read once per KV
// head).  Each thread issues all of its loads before consuming any of them; workgroups are
// small (256 threads) so that several of them overlap on a compute unit and the memory
// pipeline never drains between them.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

typedef uint32_t nt_u32x4 __attribute__((ext_vector_type(4)));
constexpr int64_t kScoreNtStoreBytes = 16 << 20;  // score arrays from this size on bypass the caches
constexpr int kScoreThreads = 256;
constexpr int kLoadsPerThread = 4;

struct ScoreArgs {
  const void* q_imp;
  const void* Kimp;
  float* scores;
  int64_t N;
  int64_t ki_stride_b, ki_stride_h, ki_stride_n;
  int64_t score_stride;
  int32_t Hq;
  float scale;
  // Large score arrays are stored non-temporally: the selection then reads them from further
  // away (C3: score + select 47.0 -> 48.8 us), but their write-back no longer competes with the
  // gathers of the attention kernel that follows (C3: 95.5 -> 86.1 us inside the step, the step
  // 142.5 -> 135.0 us).  Small ones stay in the caches for the selection (C2: 34.5 against 35.4 us).
  int32_t nt_store;
};

template <typename T, int DIMP, int G>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(ScoreArgs a) {
  constexpr int EPL = Pack16<T>::kElts;      // elements per lane (one 128-bit load)
  constexpr int LPR = DIMP / EPL;            // lanes per projected row
  constexpr int RPP = kScoreThreads / LPR;   // rows per pass of the workgroup
  constexpr int RW = RPP * kLoadsPerThread;  // rows per workgroup
  static_assert(LPR >= 1 && LPR <= 16 && (LPR & (LPR - 1)) == 0, "row must span 1..16 lanes");

  const int tid = threadIdx.x;
  const int part = tid % LPR;
  const int rsub = tid / LPR;
  const int b = blockIdx.z;
  const int hkv = blockIdx.y;
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RW;

  const T* kbase = static_cast<const T*>(a.Kimp) + b * a.ki_stride_b + hkv * a.ki_stride_h + part * EPL;

  // issue every load of this thread first (kept packed until used)
  typename Pack16<T>::Raw kraw[kLoadsPerThread];
#pragma unroll
  for (int i = 0; i < kLoadsPerThread; ++i) {
    int64_t row = row0 + i * RPP + rsub;
    row = row < a.N ? row : a.N - 1;  // clamp: the result of a clamped row is not stored
    {
      // the projected keys are streamed once per step: a non-temporal load keeps them from
      // displacing the scores (which the selection reads next) in the caches
      const nt_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(kbase + row * a.ki_stride_n));
      __builtin_memcpy(&kraw[i], &t, 16);
    }
  }

  // this lane's slice of the g importance queries
  float qv[G][EPL];
  const T* qbase = static_cast<const T*>(a.q_imp) + (static_cast<int64_t>(b) * a.Hq + hkv * G) * DIMP + part * EPL;
#pragma unroll
  for (int hh = 0; hh < G; ++hh) Pack16<T>::load(qbase + hh * DIMP, qv[hh]);

  // scores of the workgroup's RW rows for the g heads, staged in LDS so that they leave as
  // full 128-bit stores (1 KiB per wave instruction) instead of 64-byte pieces
  __shared__ float s_out[G][RW];
#pragma unroll
  for (int i = 0; i < kLoadsPerThread; ++i) {
    float kf[EPL];
    Pack16<T>::unpack(kraw[i], kf);
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) s = fmaf(qv[hh][e], kf[e], s);
      s = group_allreduce_sum<LPR>(s) * a.scale;
      if ((hh % LPR) == part) s_out[hh][i * RPP + rsub] = s;
    }
  }
  __syncthreads();
  float* sbase = a.scores + (static_cast<int64_t>(b) * a.Hq + hkv * G) * a.score_stride + row0;
  constexpr int V4 = RW / 4;  // float4 groups per head
  for (int v = tid; v < G * V4; v += kScoreThreads) {
    const int hh = v / V4, r4 = (v % V4) * 4;
    float* dst = sbase + hh * a.score_stride + r4;
    if (row0 + r4 + 3 < a.N) {
      if (a.nt_store) {
        typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(*reinterpret_cast<const nt_f32x4*>(&s_out[hh][r4]), reinterpret_cast<nt_f32x4*>(dst));
      } else {
        *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(&s_out[hh][r4]);
      }
    } else {
      for (int c = 0; c < 4; ++c)
        if (row0 + r4 + c < a.N) dst[c] = s_out[hh][r4 + c];
    }
  }
}

// ---- bf16 with Dimp = 32 on the matrix cores ----------------------------------------------------
// The g dot products of a projected row are a (rows x 32) x (32 x g) contraction.  On the vector
// ALUs they cost about 85 instructions per wave and 16 rows, and since the workgroups of a compute
// unit wait for their loads together and then compute together, that arithmetic is not hidden
// behind the stream (C2: 2.3 us of issue per compute unit in a kernel of 6.2 us).  One
// v_mfma_f32_16x16x32_bf16 does the same: the A operand of lane (i, kb) = (lane % 16, lane / 16)
// is its 128-bit load of row i, elements 8 kb .. 8 kb + 7 -- so a wave instruction still reads 1 KiB
// of consecutive memory -- and the B operand is the same slice of importance query j = lane % 16
// (zero for j >= g).  Both operands assign their eight elements to the same k, so the sum runs over
// matching elements whatever the order inside the instruction.  Accumulator v of lane (j, kb) is
// (row 4 kb + v, head j).
typedef short mfma_bf16x8 __attribute__((ext_vector_type(8)));
typedef float mfma_f32x4 __attribute__((ext_vector_type(4)));

template <int G>
__global__ __launch_bounds__(kScoreThreads) void score_mfma_kernel(ScoreArgs a) {
  constexpr int DIMP = 32;
  constexpr int RPP = kScoreThreads / 4;     // rows per pass of the workgroup: 16 per wave
  constexpr int RW = RPP * kLoadsPerThread;  // rows per workgroup
  static_assert(G <= 16, "one MFMA column per query head of the group");
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int i16 = lane & 15, kb = lane >> 4;
  const int b = blockIdx.z;
  const int hkv = blockIdx.y;
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RW;
  const bf16_t* kbase = static_cast<const bf16_t*>(a.Kimp) + b * a.ki_stride_b + hkv * a.ki_stride_h + kb * 8;

  mfma_bf16x8 kraw[kLoadsPerThread];
#pragma unroll
  for (int i = 0; i < kLoadsPerThread; ++i) {
    int64_t row = row0 + i * RPP + wave * 16 + i16;
    row = row < a.N ? row : a.N - 1;  // clamp: the result of a clamped row is not stored
    const nt_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(kbase + row * a.ki_stride_n));
    __builtin_memcpy(&kraw[i], &t, 16);
  }
  mfma_bf16x8 qop = {0, 0, 0, 0, 0, 0, 0, 0};
  if (i16 < G) {
    const bf16_t* qp = static_cast<const bf16_t*>(a.q_imp) + (static_cast<int64_t>(b) * a.Hq + hkv * G + i16) * DIMP + kb * 8;
    const uint4 t = *reinterpret_cast<const uint4*>(qp);
    __builtin_memcpy(&qop, &t, 16);
  }

  __shared__ __attribute__((aligned(16))) float s_out[G][RW];
#pragma unroll
  for (int i = 0; i < kLoadsPerThread; ++i) {
    mfma_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kraw[i], qop, acc, 0, 0, 0);
    if (i16 < G) {
      const float4 o = make_float4(acc[0] * a.scale, acc[1] * a.scale, acc[2] * a.scale, acc[3] * a.scale);
      *reinterpret_cast<float4*>(&s_out[i16 < G ? i16 : 0][i * RPP + wave * 16 + 4 * kb]) = o;
    }
  }
  __syncthreads();
  float* sbase = a.scores + (static_cast<int64_t>(b) * a.Hq + hkv * G) * a.score_stride + row0;
  constexpr int V4 = RW / 4;  // float4 groups per head
  for (int v = tid; v < G * V4; v += kScoreThreads) {
    const int hh = v / V4, r4 = (v % V4) * 4;
    float* dst = sbase + hh * a.score_stride + r4;
    if (row0 + r4 + 3 < a.N) {
      if (a.nt_store) {
        typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(*reinterpret_cast<const nt_f32x4*>(&s_out[hh][r4]), reinterpret_cast<nt_f32x4*>(dst));
      } else {
        *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(&s_out[hh][r4]);
      }
    } else {
      for (int c = 0; c < 4; ++c)
        if (row0 + r4 + c < a.N) dst[c] = s_out[hh][r4 + c];
    }
  }
}

template <typename T, int DIMP, int G>
tb_status launch_tdg(const ScoreLaunch& L, hipStream_t st) {
  const tb_cache_desc& d = *L.desc;
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int RW = kScoreThreads / (DIMP / EPL) * kLoadsPerThread;
  ScoreArgs a;
  a.q_imp = L.q_imp;
  a.Kimp = L.Kimp;
  a.scores = L.scores;
  a.N = d.N;
  a.ki_stride_b = d.ki_stride_b;
  a.ki_stride_h = d.ki_stride_h;
  a.ki_stride_n = d.ki_stride_n;
  a.score_stride = L.score_stride;
  a.Hq = d.Hq;
  a.scale = L.scale;
  a.nt_store = static_cast<int64_t>(d.B) * d.Hq * d.N * 4 >= kScoreNtStoreBytes ? 1 : 0;
  if (d.N == 0) return TB_OK;
  dim3 grid(static_cast<unsigned>((d.N + RW - 1) / RW), d.Hkv, d.B);
  if constexpr (std::is_same<T, bf16_t>::value && DIMP == 32) {
    static_assert(RW == kScoreThreads / 4 * kLoadsPerThread, "both kernels cut the rows alike");
    hipLaunchKernelGGL((score_mfma_kernel<G>), grid, dim3(kScoreThreads), 0, st, a);
  } else {
    hipLaunchKernelGGL((score_kernel<T, DIMP, G>), grid, dim3(kScoreThreads), 0, st, a);
  }
  return hip_status(hipGetLastError());
}

template <typename T, int DIMP>
tb_status launch_td(const ScoreLaunch& L, hipStream_t st) {
  switch (L.desc->Hq / L.desc->Hkv) {
    case 1: return launch_tdg<T, DIMP, 1>(L, st);
    case 2: return launch_tdg<T, DIMP, 2>(L, st);
    case 4: return launch_tdg<T, DIMP, 4>(L, st);
    case 8: return launch_tdg<T, DIMP, 8>(L, st);
    default: return TB_ERR_UNSUPPORTED;
  }
}

template <typename T>
tb_status launch_t(const ScoreLaunch& L, hipStream_t st) {
  switch (L.desc->Dimp) {
    case 16: return launch_td<T, 16>(L, st);
    case 32: return launch_td<T, 32>(L, st);
    case 64: return launch_td<T, 64>(L, st);
    default: return TB_ERR_UNSUPPORTED;
  }
}

}  // namespace

tb_status launch_score(const ScoreLaunch& L, hipStream_t st) {
  return L.desc->dtype == TB_F32 ? launch_t<float>(L, st) : launch_t<bf16_t>(L, st);
}

}  // namespace tb
