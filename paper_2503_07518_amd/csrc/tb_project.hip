// Key-cache projection K_imp = K W: rows [n_begin, n_end) of every (b, kv-head).
//
// Three forms.  project_rows_kernel takes up to four rows (the append of a decode step) with one
// wave per row.  project_kernel serves every shape:
// a workgroup projects a tile of 64 cache rows, W (D x Dimp) and the K tile are staged in LDS as
// fp32, 64 columns of the head dimension per round; thread (row, quarter) accumulates Dimp/4
// adjacent outputs in fp32 and rounds once (round to nearest even) to the storage type.
// project_mfma_kernel is the batched form for bf16 with Dimp = 16 or 32 (a window of appended rows,
// or the whole cache after prefill) on the matrix cores.
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
  int32_t tiles_per_wave;  // matrix-core form only
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

// ---- batched form for bf16 with Dimp = 16 or 32 on the matrix cores ---------------------------------
// The projection of many rows is a (rows x D) x (D x 32) contraction with 25 flop per byte:
// above what the plain fp32 FMA path sustains, so it goes through v_mfma_f32_32x32x8_bf16_1k.
// A wave projects tiles of 32 cache rows: the tile is loaded with coalesced 128-bit loads,
// passed through a padded LDS buffer into the MFMA operand layout (lane (i, kh) supplies row i,
// k = 8s + 4kh .. +3 of step s), W is transposed into LDS once per workgroup and each lane
// keeps its column's operands in registers for all tiles.  fp32 accumulators, one RNE rounding.
typedef short mfma_bf16x4 __attribute__((ext_vector_type(4)));
typedef float mfma_f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a 128-bit load kept as a plain vector
constexpr int kMfmaThreads = 256;
constexpr int kMfmaWaves = kMfmaThreads / kWave;
constexpr int kMfmaRowsPerWave = 32;                         // one MFMA tile
constexpr int kMfmaMaxTilesPerWave = 4;
constexpr int kMfmaMinRows = 2048;                           // below this the plain form is used
constexpr int kMfmaTargetWgs = 2048;                         // shorten the waves' spans to reach this

// DIMP = 16 runs the same 32-column tile with the upper 16 columns of W zero (twice the matrix
// work of what is needed, which the memory-bound kernel does not notice) and stores the lower 16.
template <int D, int DIMP>
__global__ __launch_bounds__(kMfmaThreads) void project_mfma_kernel(ProjectArgs a) {
  static_assert(DIMP == 16 || DIMP == 32, "the MFMA tile has 32 columns");
  constexpr int KSTEPS = D / 8;
  constexpr int PITCH = D * 2 + 16;         // bytes per staged row (padded against bank conflicts)
  constexpr int OPITCH = 32 * 2 + 16;       // bytes per row of the rounded output tile
  constexpr int LPR = D * 2 / 16;           // lanes per row in the coalesced load
  constexpr int RPI = kWave / LPR;          // rows per load instruction
  constexpr int NLD = 32 / RPI;             // load instructions per tile
  __shared__ __attribute__((aligned(16))) unsigned char s_k[kMfmaWaves][32 * PITCH];
  __shared__ __attribute__((aligned(16))) uint16_t s_wt[32][D + 4];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int b = blockIdx.z, h = blockIdx.y;
  const int col = lane & 31, kh = lane >> 5;

  const uint16_t* w = static_cast<const uint16_t*>(a.W) + (a.per_head_w ? static_cast<int64_t>(h) * D * DIMP : 0);
  for (int i = tid; i < D * DIMP; i += kMfmaThreads) s_wt[i % DIMP][i / DIMP] = w[i];
  if (DIMP < 32)
    for (int i = tid; i < D * (32 - DIMP); i += kMfmaThreads) s_wt[DIMP + i / D][i % D] = 0;
  __syncthreads();
  mfma_bf16x4 bop[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) bop[s] = *reinterpret_cast<const mfma_bf16x4*>(&s_wt[col][8 * s + 4 * kh]);

  const uint16_t* kb = static_cast<const uint16_t*>(a.K) + b * a.k_stride_b + h * a.k_stride_h;
  uint16_t* ob = static_cast<uint16_t*>(a.Kimp) + b * a.ki_stride_b + h * a.ki_stride_h;
  unsigned char* tile = s_k[wave];
  const int64_t wave_row0 =
      a.n_begin + (static_cast<int64_t>(blockIdx.x) * kMfmaWaves + wave) * kMfmaRowsPerWave * a.tiles_per_wave;
  const int lrow = lane / LPR;                                  // row of this lane within a load
  const uint16_t* kl = kb + (lane % LPR) * 8;                   // its 16-byte piece of the row
#define TB_LOAD_TILE(ROW0)                                                        \
  _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                               \
    int64_t row = (ROW0) + j * RPI + lrow;                                        \
    row = row < a.n_end ? row : a.n_end - 1; /* computed and dropped */           \
    v[j] = *reinterpret_cast<const u32x4*>(kl + row * a.k_stride_n);              \
  }
  if (wave_row0 >= a.n_end) return;  // the same for the whole wave (no barrier follows)
  u32x4 v[NLD];
  TB_LOAD_TILE(wave_row0)
  for (int t = 0; t < a.tiles_per_wave; ++t) {
    const int64_t row0 = wave_row0 + t * 32;
    if (row0 >= a.n_end) break;
#pragma unroll
    for (int j = 0; j < NLD; ++j)
      *reinterpret_cast<u32x4*>(tile + (j * RPI + lrow) * PITCH + (lane % LPR) * 16) = v[j];
    // the next tile's rows are on their way while this one is multiplied
    if (t + 1 < a.tiles_per_wave) { TB_LOAD_TILE(row0 + 32) }  // clamped rows: always in bounds
    mfma_f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      const mfma_bf16x4 aop = *reinterpret_cast<const mfma_bf16x4*>(tile + col * PITCH + (8 * s + 4 * kh) * 2);
      acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(aop, bop[s], acc, 0, 0, 0);
    }
    // accumulator i of lane (col, kh) is output (row = 8*(i/4) + 4*kh + i%4, column col); the
    // rounded tile goes back through LDS (the wave's own buffer, free again once the operands
    // are read: LDS operations of a wave complete in order) and leaves as 128-bit stores
#pragma unroll
    for (int i = 0; i < 16; ++i)
      *reinterpret_cast<uint16_t*>(tile + (8 * (i / 4) + 4 * kh + (i % 4)) * OPITCH + col * 2) = f32_to_bf16_rne(acc[i]);
    constexpr int PARTS = DIMP * 2 / 16;  // 128-bit pieces of an output row
#pragma unroll
    for (int j = 0; j < 32 * PARTS / kWave; ++j) {
      const int c = lane + kWave * j, r = c / PARTS, part = c % PARTS;
      const uint4 o = *reinterpret_cast<const uint4*>(tile + r * OPITCH + part * 16);
      if (row0 + r < a.n_end) *reinterpret_cast<uint4*>(ob + (row0 + r) * a.ki_stride_n + part * 8) = o;
    }
  }
#undef TB_LOAD_TILE
}

// ---- a few rows (the append of a decode step): one wave per cache row, no LDS, no barrier.
// Lane l accumulates output column l % DIMP over the slice l / DIMP of the head dimension (W rows
// are read coalesced, the K element is the same for all lanes of a slice); the slices are then
// added across lanes.  The whole chain is two dependent loads deep.
template <typename T, int D, int DIMP>
__global__ __launch_bounds__(kWave) void project_rows_kernel(ProjectArgs a) {
  constexpr int SLICES = kWave / DIMP;  // 4, 2 or 1 lanes per output column
  constexpr int DS = D / SLICES;        // head-dimension elements per slice
  const int lane = threadIdx.x;
  const int col = lane % DIMP, slice = lane / DIMP;
  const int b = blockIdx.z, h = blockIdx.y;
  const int64_t row = a.n_begin + blockIdx.x;
  const T* w = static_cast<const T*>(a.W) + (a.per_head_w ? static_cast<int64_t>(h) * D * DIMP : 0) +
               static_cast<int64_t>(slice) * DS * DIMP + col;
  const T* k = static_cast<const T*>(a.K) + b * a.k_stride_b + h * a.k_stride_h + row * a.k_stride_n + slice * DS;
  float acc = 0.f;
#pragma unroll 16
  for (int d = 0; d < DS; ++d) acc = fmaf(to_float(k[d]), to_float(w[static_cast<int64_t>(d) * DIMP]), acc);
#pragma unroll
  for (int off = DIMP; off < kWave; off <<= 1) acc += __shfl_xor(acc, off, kWave);
  if (slice == 0) {
    T* o = static_cast<T*>(a.Kimp) + b * a.ki_stride_b + h * a.ki_stride_h + row * a.ki_stride_n + col;
    store_elt(o, acc);
  }
}

template <typename T, int D, int DIMP>
tb_status launch_tdd(const tb_cache_desc& d, ProjectArgs a, hipStream_t st) {
  const int64_t rows = a.n_end - a.n_begin;
  if (rows <= 4) {
    dim3 grid(static_cast<unsigned>(rows), d.Hkv, d.B);
    hipLaunchKernelGGL((project_rows_kernel<T, D, DIMP>), grid, dim3(kWave), 0, st, a);
    return hip_status(hipGetLastError());
  }
  if constexpr (std::is_same<T, bf16_t>::value && (DIMP == 16 || DIMP == 32)) {
    if (rows >= kMfmaMinRows) {  // batched projection: enough rows to fill the matrix cores
      int tiles = kMfmaMaxTilesPerWave;
      auto wgs = [&](int t) {
        const int64_t per_wg = static_cast<int64_t>(kMfmaWaves) * kMfmaRowsPerWave * t;
        return (rows + per_wg - 1) / per_wg;
      };
      while (tiles > 1 && wgs(tiles) * d.Hkv * d.B < kMfmaTargetWgs) tiles >>= 1;
      a.tiles_per_wave = tiles;
      dim3 grid(static_cast<unsigned>(wgs(tiles)), d.Hkv, d.B);
      hipLaunchKernelGGL((project_mfma_kernel<D, DIMP>), grid, dim3(kMfmaThreads), 0, st, a);
      return hip_status(hipGetLastError());
    }
  }
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
  a.tiles_per_wave = 1;
  return d->dtype == TB_F32 ? launch_t<float>(*d, a, st) : launch_t<bf16_t>(*d, a, st);
}

}  // namespace tb
