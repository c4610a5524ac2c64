// Merge attention (Appendix B, Equation 4): bandwidth-bound streaming kernel.
//
// Every thread owns one 16-byte slice of one output row and reads the matching
// slice of each of the n_parts partial outputs exactly once, so the HBM traffic
// is the algorithmic minimum: n_parts * (row bytes + 4) in, row bytes (+4) out.
// The n_parts loads of a thread are independent and issued back to back; the
// LSE values of a row are read by all threads of the row (one cache line).
#include "cp_common.h"

namespace cp {
namespace {

struct MergePtrs {
  const void* out[CP_MAX_PARTS];
  const float* lse[CP_MAX_PARTS];
};

template <typename TP, int VEC>
__device__ __forceinline__ void load_vec(const TP* p, float (&x)[VEC]);

template <>
__device__ __forceinline__ void load_vec<float, 4>(const float* p, float (&x)[4]) {
  const floatx4_t t = __builtin_nontemporal_load((const floatx4_t*)p);
  x[0] = t[0]; x[1] = t[1]; x[2] = t[2]; x[3] = t[3];
}
template <>
__device__ __forceinline__ void load_vec<bf16_t, 8>(const bf16_t* p, float (&x)[8]) {
  const bf16x8_t t = __builtin_nontemporal_load((const bf16x8_t*)p);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = static_cast<float>(t[i]);
}

template <typename TO, int VEC>
__device__ __forceinline__ void store_vec(TO* p, const float (&x)[VEC]);
template <>
__device__ __forceinline__ void store_vec<float, 4>(float* p, const float (&x)[4]) {
  floatx4_t t = {x[0], x[1], x[2], x[3]};
  *(floatx4_t*)p = t;
}
template <>
__device__ __forceinline__ void store_vec<float, 8>(float* p, const float (&x)[8]) {
  floatx4_t a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
  ((floatx4_t*)p)[0] = a;
  ((floatx4_t*)p)[1] = b;
}
template <>
__device__ __forceinline__ void store_vec<bf16_t, 4>(bf16_t* p, const float (&x)[4]) {
  bf16x4_t t;
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = static_cast<bf16_t>(x[i]);
  *(bf16x4_t*)p = t;
}
template <>
__device__ __forceinline__ void store_vec<bf16_t, 8>(bf16_t* p, const float (&x)[8]) {
  bf16x8_t t;
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = static_cast<bf16_t>(x[i]);
  *(bf16x8_t*)p = t;
}

// NP > 0: compile-time part count (fully unrolled); NP == 0: run-time count.
// STRIDED: partials are parts_out + s * stride (split-KV scratch) instead of pointers.
template <typename TP, typename TO, int VEC, int NP, bool STRIDED>
__global__ __launch_bounds__(256) void merge_kernel(MergePtrs ptrs, const float* parts_out,
                                                     const float* parts_lse,
                                                     int64_t part_stride_rows, int n_parts_rt,
                                                     int64_t rows, int head_dim,
                                                     TO* __restrict__ out,
                                                     float* __restrict__ lse_out) {
  const int n_parts = NP > 0 ? NP : n_parts_rt;
  const int vec_per_row = head_dim / VEC;
  const int64_t n_vec = rows * vec_per_row;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n_vec;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = idx / vec_per_row;
    const int col = (int)(idx - row * vec_per_row) * VEC;

    // With a compile-time part count the LSE values stay in registers; with a run-time
    // count they are read twice (a per-thread array indexed at run time would live in scratch).
    float lmax = -INFINITY;
    float lv[NP > 0 ? NP : 1];
#pragma unroll
    for (int s = 0; s < n_parts; ++s) {
      const float x = STRIDED ? parts_lse[s * part_stride_rows + row] : ptrs.lse[s][row];
      if (NP > 0) lv[NP > 0 ? s : 0] = x;
      lmax = fmaxf(lmax, x);
    }
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    float den = 0.f;
    if constexpr (STRIDED && NP > 0 && NP <= 16) {
      // Split-KV scratch of one call: few rows, so the kernel is bound by latency, not by
      // bandwidth. Every row of the scratch is written (finite zeros when empty), so all NP
      // loads are issued at once, next to the LSE loads, and the arithmetic is branch-free
      // (a branch on the weights would pull the loads behind the wait for the LSE values).
      float xs[NP][VEC];
#pragma unroll
      for (int s = 0; s < NP; ++s)
        load_vec<TP, VEC>((const TP*)(parts_out + (s * part_stride_rows + row) * head_dim) + col,
                          xs[s]);
      __builtin_amdgcn_sched_barrier(0);  // keep the NP loads together, ahead of the arithmetic
      const bool any = lmax != -INFINITY;
#pragma unroll
      for (int s = 0; s < NP; ++s) {
        const float w = any ? __expf(lv[s] - lmax) : 0.f;  // exp(-inf) = 0 for empty partials
        den += w;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, xs[s][i], acc[i]);
      }
      const float inv = any ? 1.f / den : 0.f;
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] *= inv;
    } else if (lmax != -INFINITY) {
#pragma unroll
      for (int s = 0; s < n_parts; ++s) {
        const float x = NP > 0 ? lv[NP > 0 ? s : 0]
                               : (STRIDED ? parts_lse[s * part_stride_rows + row] : ptrs.lse[s][row]);
        const float w = __expf(x - lmax);  // exp(-inf) = 0 for empty partials
        den += w;
        // split-KV scratch rows are always written (zeros when empty), so their loads need
        // not wait for the weights; caller-supplied partials with zero weight are not read
        if (STRIDED || w != 0.f) {
          const TP* p = STRIDED ? (const TP*)(parts_out + (s * part_stride_rows + row) * head_dim)
                                : (const TP*)ptrs.out[s] + row * head_dim;
          float x4[VEC];
          load_vec<TP, VEC>(p + col, x4);
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, x4[i], acc[i]);
        }
      }
      const float inv = 1.f / den;
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] *= inv;
    }
    store_vec<TO, VEC>(out + row * head_dim + col, acc);
    if (lse_out != nullptr && col == 0)
      lse_out[row] = lmax == -INFINITY ? -INFINITY : lmax + __logf(den);
  }
}

template <typename TP, typename TO, int VEC, bool STRIDED>
int launch_np(const MergePtrs& ptrs, const float* parts_out, const float* parts_lse,
              int64_t stride, int n_parts, int64_t rows, int head_dim, void* out, float* lse_out,
              hipStream_t stream) {
  const int64_t n_vec = rows * (head_dim / VEC);
  if (n_vec == 0) return CP_OK;
  // Small merges (the split partials of a decode step) are latency-bound: one wavefront per
  // workgroup spreads them over every CU instead of a quarter of them.
#ifndef CP_MERGE_SMALL_VEC
#define CP_MERGE_SMALL_VEC (256 * 256)
#endif
  const int threads = n_vec <= CP_MERGE_SMALL_VEC ? 64 : 256;
  int64_t blocks = (n_vec + threads - 1) / threads;
  const int64_t cap = 256 * 32;  // grid-stride beyond 32 workgroups per CU
  if (blocks > cap) blocks = cap;
#define CP_MERGE_LAUNCH(NP)                                                                   \
  hipLaunchKernelGGL((merge_kernel<TP, TO, VEC, NP, STRIDED>), dim3((unsigned)blocks),        \
                     dim3(threads), 0, stream, ptrs, parts_out, parts_lse, stride, n_parts,   \
                     rows, head_dim, (TO*)out, lse_out)
  switch (n_parts) {
    case 2: CP_MERGE_LAUNCH(2); break;
    case 4: CP_MERGE_LAUNCH(4); break;
    case 8: CP_MERGE_LAUNCH(8); break;
    case 16: CP_MERGE_LAUNCH(16); break;
    case 32: if (STRIDED) { CP_MERGE_LAUNCH(32); } else { CP_MERGE_LAUNCH(0); } break;
    case 64: if (STRIDED) { CP_MERGE_LAUNCH(64); } else { CP_MERGE_LAUNCH(0); } break;
    default: CP_MERGE_LAUNCH(0); break;
  }
#undef CP_MERGE_LAUNCH
  return check_launch();
}

}  // namespace

int launch_merge(int64_t rows, int32_t head_dim, int32_t n_parts, const void* const* outs,
                 const float* const* lses, int32_t part_dtype, void* out, int32_t out_dtype,
                 float* lse_out, hipStream_t stream) {
  MergePtrs ptrs;
  for (int s = 0; s < CP_MAX_PARTS; ++s) {
    ptrs.out[s] = s < n_parts ? outs[s] : nullptr;
    ptrs.lse[s] = s < n_parts ? lses[s] : nullptr;
  }
  if (part_dtype == CP_FP32) {
    if (out_dtype == CP_FP32)
      return launch_np<float, float, 4, false>(ptrs, nullptr, nullptr, 0, n_parts, rows,
                                               head_dim, out, lse_out, stream);
    return launch_np<float, bf16_t, 4, false>(ptrs, nullptr, nullptr, 0, n_parts, rows, head_dim,
                                              out, lse_out, stream);
  }
  if (out_dtype == CP_FP32)
    return launch_np<bf16_t, float, 8, false>(ptrs, nullptr, nullptr, 0, n_parts, rows, head_dim,
                                              out, lse_out, stream);
  return launch_np<bf16_t, bf16_t, 8, false>(ptrs, nullptr, nullptr, 0, n_parts, rows, head_dim,
                                             out, lse_out, stream);
}

int launch_merge_strided(int64_t rows, int32_t head_dim, int32_t n_parts, const float* parts_out,
                         const float* parts_lse, int64_t part_stride_rows, void* out,
                         int32_t out_dtype, float* lse_out, hipStream_t stream) {
  MergePtrs ptrs = {};
  if (out_dtype == CP_FP32)
    return launch_np<float, float, 4, true>(ptrs, parts_out, parts_lse, part_stride_rows,
                                            n_parts, rows, head_dim, out, lse_out, stream);
  return launch_np<float, bf16_t, 4, true>(ptrs, parts_out, parts_lse, part_stride_rows, n_parts,
                                           rows, head_dim, out, lse_out, stream);
}

}  // namespace cp
