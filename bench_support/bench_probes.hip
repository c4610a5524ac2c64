// Yardsticks for bench.py (not part of libcp_attn and not a step of the paper's method):
//   bench_probe_mfma_rate  what the matrix pipe sustains on this part for given operand
//                          values: a loop of independent bf16 MFMAs on register operands and
//                          nothing else. With N(0,1) operands the part draws more power than
//                          with zeros and settles at a lower clock.
//   bench_probe_hbm_read   what one launch that only streams a buffer once achieves, launch
//                          ramp and tail included: the yardstick for the split-KV decode kernel
//                          beside the published HBM peak.
// Both return 0, or a negative value for bad arguments (-1 null pointer, -2 bad size,
// -5 launch failure, -6 misaligned buffer); work is enqueued on `hip_stream`.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#define BENCH_PROBE_OPERAND_BYTES 65536

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

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
  constexpr int DEPTH = 8;
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

extern "C" int bench_probe_mfma_rate(const void* operands, int32_t iters, int32_t n_workgroups,
                                  void* sink, double* flop_out, void* hip_stream) {
  static_assert(BENCH_PROBE_OPERAND_BYTES == 512 * 8 * sizeof(bf16x8_t), "operand block");
  if (operands == nullptr || sink == nullptr || flop_out == nullptr) return -1;
  if (iters < 1 || n_workgroups < 1) return -2;
  hipLaunchKernelGGL(mfma_rate_probe_kernel, dim3(n_workgroups), dim3(512), 0,
                     (hipStream_t)hip_stream, (const bf16x8_t*)operands, (float*)sink, iters);
  if (hipGetLastError() != hipSuccess) return -5;
  // 8 wavefronts x 16 MFMAs per iteration, 2 * 32 * 32 * 16 operations each
  *flop_out = (double)n_workgroups * 8.0 * (double)iters * 16.0 * 32768.0;
  return 0;
}

extern "C" int bench_probe_hbm_read(const void* buffer, size_t bytes, int32_t n_workgroups,
                                 void* sink, void* hip_stream) {
  if (buffer == nullptr || sink == nullptr) return -1;
  if (n_workgroups < 1 || bytes < 16 || bytes % 16 != 0) return -2;
  if (((uintptr_t)buffer & 15u) != 0) return -6;
  hipLaunchKernelGGL(hbm_read_probe_kernel, dim3(n_workgroups), dim3(256), 0,
                     (hipStream_t)hip_stream, (const uint4*)buffer, (int64_t)(bytes / 16),
                     (uint32_t*)sink);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}
