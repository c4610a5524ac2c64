// Measurement support: what the matrix pipe sustains on this part for given operand values.
// A loop of independent bf16 MFMAs on register operands, nothing else: the ceiling any
// MFMA-bound kernel is measured against next to the published peak. With N(0,1) operands the
// part draws more power than with zeros and settles at a lower clock.
#include "cp_common.h"

namespace cp {
namespace {

__global__ __launch_bounds__(512) void mfma_rate_probe_kernel(const bf16x8_t* __restrict__ in,
                                                              float* __restrict__ sink,
                                                              int iters) {
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = in[threadIdx.x + 512 * i];
    b[i] = in[threadIdx.x + 512 * (4 + i)];
  }
  floatx16_t o[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 16; ++m)
      o[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m & 3], b[(m >> 2) & 3], o[m & 3], 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += o[c][i];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// What one launch that does nothing but read `n_chunks` 16-byte chunks once sustains: every
// thread walks the buffer with a grid-wide stride, non-temporal loads, eight in flight, and
// folds what it read into one word so that no load can be dropped.
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const uint4* __restrict__ in,
                                                             int64_t n_chunks,
                                                             uint32_t* __restrict__ sink) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t acc = 0;
#ifndef CP_PROBE_DEPTH
#define CP_PROBE_DEPTH 8
#endif
  constexpr int DEPTH = CP_PROBE_DEPTH;
  for (; i + (DEPTH - 1) * stride < n_chunks; i += DEPTH * stride) {
    uint4 t[DEPTH];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
      t[u] = __builtin_bit_cast(uint4,
                                __builtin_nontemporal_load((const u32x4_t*)(in + i + u * stride)));
    }
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) acc ^= t[u].x ^ t[u].y ^ t[u].z ^ t[u].w;
  }
  for (; i < n_chunks; i += stride) {
    const uint4 t = in[i];
    acc ^= t.x ^ t.y ^ t.z ^ t.w;
  }
  sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

}  // namespace
}  // namespace cp

extern "C" int cp_probe_mfma_rate(const void* operands, int32_t iters, int32_t n_workgroups,
                                  void* sink, double* flop_out, void* hip_stream) {
  static_assert(CP_PROBE_OPERAND_BYTES == 512 * 8 * sizeof(cp::bf16x8_t), "operand block");
  if (operands == nullptr || sink == nullptr || flop_out == nullptr) return CP_ERR_NULL;
  if (iters < 1 || n_workgroups < 1) return CP_ERR_SHAPE;
  hipLaunchKernelGGL(cp::mfma_rate_probe_kernel, dim3(n_workgroups), dim3(512), 0,
                     (hipStream_t)hip_stream, (const cp::bf16x8_t*)operands, (float*)sink, iters);
  if (cp::check_launch() != CP_OK) return CP_ERR_LAUNCH;
  // 8 wavefronts x 16 MFMAs per iteration, 2 * 32 * 32 * 16 operations each
  *flop_out = (double)n_workgroups * 8.0 * (double)iters * 16.0 * 32768.0;
  return CP_OK;
}

extern "C" int cp_probe_hbm_read(const void* buffer, size_t bytes, int32_t n_workgroups,
                                 void* sink, void* hip_stream) {
  if (buffer == nullptr || sink == nullptr) return CP_ERR_NULL;
  if (n_workgroups < 1 || bytes < 16 || bytes % 16 != 0) return CP_ERR_SHAPE;
  if (((uintptr_t)buffer & 15u) != 0) return CP_ERR_ALIGN;
  hipLaunchKernelGGL(cp::hbm_read_probe_kernel, dim3(n_workgroups), dim3(256), 0,
                     (hipStream_t)hip_stream, (const uint4*)buffer, (int64_t)(bytes / 16),
                     (uint32_t*)sink);
  return cp::check_launch();
}
