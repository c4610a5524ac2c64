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
