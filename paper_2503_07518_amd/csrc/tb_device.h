// Device-side helpers shared by the HIP kernels of the TokenButler decode hot path (gfx950,
// wave64).  Nothing here is used by, or shared with, the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace tb {

constexpr int kWave = 64;

// Storage element types.  bf16 is handled as raw bits: the upper half of an fp32.
struct bf16_t {
  uint16_t bits;
};

template <typename T>
struct Pack16;  // one 16-byte vector of T, unpacked to fp32

template <>
struct Pack16<float> {
  static constexpr int kElts = 4;
  using Raw = float4;
  __device__ static inline Raw load_raw(const void* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static inline void unpack(const Raw& v, float (&f)[4]) {
    f[0] = v.x;
    f[1] = v.y;
    f[2] = v.z;
    f[3] = v.w;
  }
  __device__ static inline void load(const float* p, float (&f)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    f[0] = v.x;
    f[1] = v.y;
    f[2] = v.z;
    f[3] = v.w;
  }
};

template <>
struct Pack16<bf16_t> {
  static constexpr int kElts = 8;
  using Raw = uint4;
  __device__ static inline Raw load_raw(const void* p) { return *reinterpret_cast<const uint4*>(p); }
  __device__ static inline void unpack(const Raw& v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    f[4] = __uint_as_float(v.z << 16);
    f[5] = __uint_as_float(v.z & 0xFFFF0000u);
    f[6] = __uint_as_float(v.w << 16);
    f[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
  __device__ static inline void load(const bf16_t* p, float (&f)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    f[4] = __uint_as_float(v.z << 16);
    f[5] = __uint_as_float(v.z & 0xFFFF0000u);
    f[6] = __uint_as_float(v.w << 16);
    f[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
};

__device__ inline float to_float(float x) { return x; }
__device__ inline float to_float(bf16_t x) { return __uint_as_float(static_cast<uint32_t>(x.bits) << 16); }

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t b = __float_as_uint(f);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((b >> 16) | 0x0040u);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return static_cast<uint16_t>(b >> 16);
}

__device__ inline void store_elt(float* p, float v) { *p = v; }
__device__ inline void store_elt(bf16_t* p, float v) { p->bits = f32_to_bf16_rne(v); }

// Order-preserving map from a score to an unsigned key: a larger score gives a larger key.
// NaN ranks with -inf and -0 equals +0 (selection policy).  The smallest key a real score can
// produce is 0x007FFFFF (-inf), so key 0 is free to mark "not a candidate".
__device__ inline uint32_t score_key(float s) {
  // IEEE maxNum returns the operand that is a number, so NaN becomes -inf; adding +0 turns -0
  // into +0 and changes nothing else (subnormals are kept: fp32 denormal mode is "preserve")
  const uint32_t b = __float_as_uint(fmaxf(s, -__builtin_inff()) + 0.0f);
  // flip all bits of negatives, only the sign bit of non-negatives
  return b ^ (static_cast<uint32_t>(static_cast<int32_t>(b) >> 31) | 0x80000000u);
}

__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }
// Index of the wave inside its workgroup, as a value the compiler knows to be the same in every
// lane: what is derived from it (the wave's span of a row, its LDS region, branches on them)
// stays in scalar registers and scalar branches.
__device__ inline int wave_id() { return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave); }

// Inclusive prefix sum across the 64 lanes of a wave (generic: LDS-crossbar shuffles).
template <typename T>
__device__ inline T wave_incl_scan(T v) {
  const int lane = lane_id();
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    T o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  return v;
}

// 32-bit inclusive prefix sum with DPP moves (stays in the VALU, no LDS traffic): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0/2 is broadcast into row
// 1/3 and the last lane of the lower half into the upper half.  Lanes whose source falls
// outside the row (or outside the enabled rows) receive 0.
__device__ inline uint32_t wave_incl_scan_u32(uint32_t v) {
  constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
  v += __builtin_amdgcn_update_dpp(0u, v, kRowShr + 1, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, kRowShr + 2, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, kRowShr + 4, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, kRowShr + 8, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, kRowBcast15, 0xA, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, kRowBcast31, 0xC, 0xF, false);
  return v;
}

// Sum over aligned groups of LANES adjacent lanes (LANES = 1..32, a power of two); every lane
// of a group receives the group's total.  The exchanges inside a row of 16 lanes are DPP moves
// (swap neighbours, swap pairs, mirror the half row, mirror the row) and stay in the VALU;
// only a 32-lane group needs one cross-row shuffle.
template <int LANES>
__device__ inline float group_allreduce_sum(float s) {
  constexpr int kQuadSwap1 = 0xB1;  // quad_perm [1,0,3,2]
  constexpr int kQuadSwap2 = 0x4E;  // quad_perm [2,3,0,1]
  constexpr int kRowHalfMirror = 0x141, kRowMirror = 0x140;
  auto dpp = [](float x, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, false));
  };
  if (LANES >= 2) s += dpp(s, std::integral_constant<int, kQuadSwap1>{});
  if (LANES >= 4) s += dpp(s, std::integral_constant<int, kQuadSwap2>{});
  if (LANES >= 8) s += dpp(s, std::integral_constant<int, kRowHalfMirror>{});
  if (LANES >= 16) s += dpp(s, std::integral_constant<int, kRowMirror>{});
  if (LANES >= 32) s += __shfl_xor(s, 16, kWave);
  return s;
}

// Exclusive prefix sum over the threads of a block of NWAVES waves (thread order).
// s_tmp needs NWAVES + 1 entries.  Ends with a barrier, so s_tmp may be reused right away
// for another scan.  `total` receives the block-wide sum.
template <int NWAVES, typename T>
__device__ inline T block_excl_scan(T v, T* s_tmp, T& total) {
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const T incl = wave_incl_scan(v);
  if (lane == kWave - 1) s_tmp[wave] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    T run = 0;
    for (int w = 0; w < NWAVES; ++w) {
      const T t = s_tmp[w];
      s_tmp[w] = run;
      run += t;
    }
    s_tmp[NWAVES] = run;
  }
  __syncthreads();
  const T base = s_tmp[wave];
  total = s_tmp[NWAVES];
  __syncthreads();
  return base + incl - v;
}

}  // namespace tb
