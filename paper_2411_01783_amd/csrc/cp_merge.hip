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
template <typename TP, typename TO, int VEC, int NP>
__global__ __launch_bounds__(256) void merge_kernel(MergePtrs ptrs, int n_parts_rt, int64_t rows,
                                                     int head_dim, TO* __restrict__ out,
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
      const float x = ptrs.lse[s][row];
      if (NP > 0) lv[NP > 0 ? s : 0] = x;
      lmax = fmaxf(lmax, x);
    }
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    float den = 0.f;
    if (lmax != -INFINITY) {
#pragma unroll
      for (int s = 0; s < n_parts; ++s) {
        const float x = NP > 0 ? lv[NP > 0 ? s : 0] : ptrs.lse[s][row];
        const float w = __expf(x - lmax);  // exp(-inf) = 0 for empty partials
        den += w;
        // a partial with zero weight is not read (its O may hold anything)
        if (w != 0.f) {
          const TP* p = (const TP*)ptrs.out[s] + row * head_dim;
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

// Split-KV scratch of one call (partials s * stride apart, every row written: finite zeros
// and LSE = -inf when a split saw nothing). Few rows, so the kernel is bound by latency, not
// by bandwidth: a thread requests the LSE values of all parts and 16 data vectors at a time
// back to back, and the arithmetic is branch-free (a branch on the weights would pull the
// loads behind the wait for the LSE values).
template <typename TO>
__global__ __launch_bounds__(64) void merge_split_kernel(const float* __restrict__ parts_out,
                                                         const float* __restrict__ parts_lse,
                                                         int64_t part_stride_rows, int n_parts,
                                                         int64_t rows, int head_dim,
                                                         TO* __restrict__ out,
                                                         float* __restrict__ lse_out) {
  constexpr int VEC = 4, BATCH = 16;
  const int vec_per_row = head_dim / VEC;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * vec_per_row) return;
  const int64_t row = idx / vec_per_row;
  const int col = (int)(idx - row * vec_per_row) * VEC;
  float lv[CP_MAX_PARTS];
#pragma unroll
  for (int s = 0; s < CP_MAX_PARTS; ++s)
    lv[s] = s < n_parts ? parts_lse[s * part_stride_rows + row] : -INFINITY;
  float acc[VEC] = {0.f, 0.f, 0.f, 0.f};
  float den = 0.f, lmax = -INFINITY;
#pragma unroll
  for (int b = 0; b < CP_MAX_PARTS / BATCH; ++b) {
    if (b * BATCH >= n_parts) break;  // uniform
    float xs[BATCH][VEC];
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      const int s = min(b * BATCH + i, n_parts - 1);  // parts past the end: weight 0 below
      load_vec<float, VEC>(parts_out + (s * part_stride_rows + row) * head_dim + col, xs[i]);
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the requests together, ahead of the arithmetic
    if (b == 0) {
#pragma unroll
      for (int s = 0; s < CP_MAX_PARTS; ++s) lmax = fmaxf(lmax, lv[s]);
    }
    const bool any = lmax != -INFINITY;
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      const float w = any ? __expf(lv[b * BATCH + i] - lmax) : 0.f;  // exp(-inf) = 0
      den += w;
#pragma unroll
      for (int c = 0; c < VEC; ++c) acc[c] = fmaf(w, xs[i][c], acc[c]);
    }
  }
  const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
  for (int c = 0; c < VEC; ++c) acc[c] *= inv;
  store_vec<TO, VEC>(out + row * head_dim + col, acc);
  if (lse_out != nullptr && col == 0)
    lse_out[row] = den > 0.f ? lmax + __logf(den) : -INFINITY;
}

template <typename TP, typename TO, int VEC>
int launch_np(const MergePtrs& ptrs, int n_parts, int64_t rows, int head_dim, void* out,
              float* lse_out, hipStream_t stream) {
  const int64_t n_vec = rows * (head_dim / VEC);
  if (n_vec == 0) return CP_OK;
  int64_t blocks = (n_vec + 255) / 256;
  const int64_t cap = 256 * 32;  // grid-stride beyond 32 workgroups per CU
  if (blocks > cap) blocks = cap;
#define CP_MERGE_LAUNCH(NP)                                                                  \
  hipLaunchKernelGGL((merge_kernel<TP, TO, VEC, NP>), dim3((unsigned)blocks), dim3(256), 0,  \
                     stream, ptrs, n_parts, rows, head_dim, (TO*)out, lse_out)
  switch (n_parts) {
    case 2: CP_MERGE_LAUNCH(2); break;
    case 4: CP_MERGE_LAUNCH(4); break;
    case 8: CP_MERGE_LAUNCH(8); break;
    case 16: CP_MERGE_LAUNCH(16); break;
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
      return launch_np<float, float, 4>(ptrs, n_parts, rows, head_dim, out, lse_out, stream);
    return launch_np<float, bf16_t, 4>(ptrs, n_parts, rows, head_dim, out, lse_out, stream);
  }
  if (out_dtype == CP_FP32)
    return launch_np<bf16_t, float, 8>(ptrs, n_parts, rows, head_dim, out, lse_out, stream);
  return launch_np<bf16_t, bf16_t, 8>(ptrs, n_parts, rows, head_dim, out, lse_out, stream);
}

constexpr int64_t kStridedStreamRows = 4096;

int launch_merge_strided(int64_t rows, int32_t head_dim, int32_t n_parts, const float* parts_out,
                         const float* parts_lse, int64_t part_stride_rows, void* out,
                         int32_t out_dtype, float* lse_out, hipStream_t stream) {
  const int64_t n_vec = rows * (head_dim / 4);
  if (n_vec == 0) return CP_OK;
  if (n_parts < 1 || n_parts > CP_MAX_PARTS || n_vec > 0x7fffffffLL * 64) return CP_ERR_SHAPE;
  // Many rows: the work is bound by bandwidth, not by latency, and the streaming kernel with
  // its compile-time part counts moves it faster (measured at 16384 rows x 4 parts: 14 us
  // here against 8 us there; with a run-time part count it is slower than this kernel).
  if (rows >= kStridedStreamRows && (n_parts == 2 || n_parts == 4 || n_parts == 8 || n_parts == 16)) {
    const void* outs[CP_MAX_PARTS];
    const float* lses[CP_MAX_PARTS];
    for (int s = 0; s < n_parts; ++s) {
      outs[s] = parts_out + (int64_t)s * part_stride_rows * head_dim;
      lses[s] = parts_lse + (int64_t)s * part_stride_rows;
    }
    return launch_merge(rows, head_dim, n_parts, outs, lses, CP_FP32, out, out_dtype, lse_out,
                        stream);
  }
  const dim3 grid((unsigned)((n_vec + 63) / 64));
  if (out_dtype == CP_FP32)
    hipLaunchKernelGGL(merge_split_kernel<float>, grid, dim3(64), 0, stream, parts_out, parts_lse,
                       part_stride_rows, n_parts, rows, head_dim, (float*)out, lse_out);
  else
    hipLaunchKernelGGL(merge_split_kernel<bf16_t>, grid, dim3(64), 0, stream, parts_out,
                       parts_lse, part_stride_rows, n_parts, rows, head_dim, (bf16_t*)out, lse_out);
  return check_launch();
}

}  // namespace cp
