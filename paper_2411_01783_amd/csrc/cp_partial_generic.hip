// fp32 vector-ALU partial attention: one wavefront per (query token, query head).
//
// Serves the shapes the MFMA kernel does not take (fp32 inputs, head_dim 64,
// packed batches). It follows Appendix B directly: scores of 64 keys at a time,
// a running maximum and denominator (online softmax), and a running weighted
// sum of values. Correctness path; not tuned.
#include "cp_common.h"

namespace cp {
namespace {

constexpr int kWaves = 4;  // wavefronts (rows) per workgroup

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

template <typename T, typename TO, int D>
__global__ __launch_bounds__(kWaves * 64) void partial_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ kv_pos,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, int batch,
    int64_t total_q, int64_t total_kv, int n_q_heads, int n_kv_heads, float scale,
    TO* __restrict__ out, float* __restrict__ lse) {
  constexpr int DPL = D / 64;  // output dims per lane
  __shared__ float q_lds[kWaves][D];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWaves + wave;  // (token, head)
  if (row >= total_q * n_q_heads) return;
  const int64_t tok = row / n_q_heads;
  const int h = (int)(row % n_q_heads);
  const int g = h / (n_q_heads / n_kv_heads);

  int64_t k0 = 0, k1 = total_kv;
  if (cu_q != nullptr) {
    int b = 0;
    while (b + 1 < batch && cu_q[b + 1] <= tok) ++b;
    k0 = cu_kv[b];
    k1 = cu_kv[b + 1];
  }
  const int32_t qp = q_pos[tok];
  for (int c = lane; c < D; c += 64) q_lds[wave][c] = to_float(q[row * D + c]);
  __builtin_amdgcn_wave_barrier();

  float m = -INFINITY, l = 0.f;
  float acc[DPL];
#pragma unroll
  for (int c = 0; c < DPL; ++c) acc[c] = 0.f;

  for (int64_t j0 = k0; j0 < k1; j0 += 64) {
    const int64_t j = j0 + lane;
    const bool vis = j < k1 && kv_pos[j] <= qp;
    float s = -INFINITY;
    if (vis) {
      const T* kj = k + (j * n_kv_heads + g) * D;
      float dot = 0.f;
#pragma unroll 8
      for (int c = 0; c < D; ++c) dot = fmaf(q_lds[wave][c], to_float(kj[c]), dot);
      s = dot * scale;
    }
    const float bm = wave_max(s);
    if (bm == -INFINITY) continue;  // whole block masked (uniform)
    const float m_new = fmaxf(m, bm);
    const float corr = (m == -INFINITY) ? 0.f : __expf(m - m_new);
    const float p = vis ? __expf(s - m_new) : 0.f;
    l = l * corr + wave_sum(p);
#pragma unroll
    for (int c = 0; c < DPL; ++c) acc[c] *= corr;
    const int nblk = (int)((k1 - j0) < 64 ? (k1 - j0) : 64);
    for (int t = 0; t < nblk; ++t) {
      const float pt = __shfl(p, t, 64);
      if (pt == 0.f) continue;  // masked key: its V is never read (uniform branch)
      const T* vj = v + ((j0 + t) * n_kv_heads + g) * D + lane * DPL;
#pragma unroll
      for (int c = 0; c < DPL; ++c) acc[c] = fmaf(pt, to_float(vj[c]), acc[c]);
    }
    m = m_new;
  }

  const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
  for (int c = 0; c < DPL; ++c) out[row * D + lane * DPL + c] = from_float<TO>(acc[c] * inv);
  if (lane == 0) lse[row] = l > 0.f ? m + __logf(l) : -INFINITY;
}

template <typename T, typename TO, int D>
int launch_t(const cp_shape& s, float scale, const void* q, const void* k, const void* v,
             const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_q,
             const int32_t* cu_kv, void* out, float* lse, hipStream_t stream) {
  const int64_t rows = s.total_q * s.n_q_heads;
  if (rows == 0) return CP_OK;
  const int64_t blocks = (rows + kWaves - 1) / kWaves;
  if (blocks > 0x7fffffffLL) return CP_ERR_SHAPE;
  hipLaunchKernelGGL((partial_generic_kernel<T, TO, D>), dim3((unsigned)blocks),
                     dim3(kWaves * 64), 0, stream, (const T*)q, (const T*)k, (const T*)v, q_pos,
                     kv_pos, cu_q, cu_kv, s.batch, s.total_q, s.total_kv, s.n_q_heads,
                     s.n_kv_heads, scale, (TO*)out, lse);
  return check_launch();
}

template <typename T, int D>
int launch_o(const cp_shape& s, float scale, const void* q, const void* k, const void* v,
             const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_q,
             const int32_t* cu_kv, void* out, float* lse, int32_t out_dtype,
             hipStream_t stream) {
  if (out_dtype == CP_FP32)
    return launch_t<T, float, D>(s, scale, q, k, v, q_pos, kv_pos, cu_q, cu_kv, out, lse, stream);
  return launch_t<T, bf16_t, D>(s, scale, q, k, v, q_pos, kv_pos, cu_q, cu_kv, out, lse, stream);
}

}  // namespace

int launch_partial_generic(const cp_shape& s, float scale, const void* q, const void* k,
                           const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                           const int32_t* cu_q, const int32_t* cu_kv, void* out, float* lse,
                           int32_t out_dtype, hipStream_t stream) {
  if (s.dtype == CP_FP32) {
    if (s.head_dim == 64)
      return launch_o<float, 64>(s, scale, q, k, v, q_pos, kv_pos, cu_q, cu_kv, out, lse,
                                 out_dtype, stream);
    return launch_o<float, 128>(s, scale, q, k, v, q_pos, kv_pos, cu_q, cu_kv, out, lse,
                                out_dtype, stream);
  }
  if (s.head_dim == 64)
    return launch_o<bf16_t, 64>(s, scale, q, k, v, q_pos, kv_pos, cu_q, cu_kv, out, lse,
                                out_dtype, stream);
  return launch_o<bf16_t, 128>(s, scale, q, k, v, q_pos, kv_pos, cu_q, cu_kv, out, lse,
                               out_dtype, stream);
}

}  // namespace cp
