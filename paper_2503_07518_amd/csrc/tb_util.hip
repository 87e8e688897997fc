// Utility kernels of libtokenbutler that are not steps of the method: the workspace fill and a
// read-stream probe used as a bandwidth calibration.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

__global__ void fill_zero_kernel(uint32_t* p, size_t words) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < words;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    p[i] = 0u;
}

// A plain read stream: every thread issues 8 non-temporal 128-bit loads 4 KiB apart (a wave
// instruction reads 1 KiB of consecutive memory) and folds them; nothing is written unless the
// fold hits one particular value.  What this reaches is the box's practical ceiling for the
// streaming kernels of the path, next to the data-sheet bandwidth.
typedef uint32_t read_u32x4 __attribute__((ext_vector_type(4)));
constexpr int kReadLoads = 8;
__global__ __launch_bounds__(256) void read_stream_kernel(const read_u32x4* p, size_t n, uint32_t* sink) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 * kReadLoads + threadIdx.x;
  read_u32x4 v[kReadLoads];
#pragma unroll
  for (int k = 0; k < kReadLoads; ++k) {
    const size_t at = i + static_cast<size_t>(k) * 256;
    v[k] = __builtin_nontemporal_load(p + (at < n ? at : 0));
  }
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < kReadLoads; ++k) s += v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  if (s == 0x9E3779B9u) sink[0] = s;
}
}  // namespace

tb_status launch_read_stream(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
  const size_t n = bytes / 16;
  if (n == 0) return TB_OK;
  const size_t blocks = (n + 256 * kReadLoads - 1) / (256 * kReadLoads);
  if (blocks > 0x7FFFFFFFu) return TB_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(read_stream_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st,
                     static_cast<const read_u32x4*>(src), n, sink);
  return hip_status(hipGetLastError());
}

tb_status launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  const size_t words = bytes / 4;
  if (words == 0) return TB_OK;
  size_t blocks = (words + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st,
                     static_cast<uint32_t*>(p), words);
  return hip_status(hipGetLastError());
}

}  // namespace tb
