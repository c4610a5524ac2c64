// Packed (variable-length) batches for the MFMA prefill kernel (Algorithm 2's fused
// variable-length inputs, Section 3.4).
//
// The prefill kernel masks with one position per token. Several sequences packed into one
// call are told apart by moving every sequence into its own position range: sequence b is
// shifted by base_b = sum over b' < b of span_b', where span_b' = 1 + the largest position
// any query or key of sequence b' carries. A key is then visible to a query iff
//   q_lo <= kv_enc <= q_hi,   q_lo = base_b,   q_hi = base_b + q_pos,   kv_enc = base_b + kv_pos,
// which is the causal mask inside the sequence and nothing across sequences. Padding keeps
// its meaning: a padded key stays at INT32_MAX, a padded query gets the empty range [0, -1].
// The shifted positions must stay below 2^31 - 1 (sum of the spans); beyond that the scan
// saturates and the later sequences see nothing.
#include "cp_common.h"

namespace cp {
namespace {

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

__global__ __launch_bounds__(256) void seq_span_kernel(const int32_t* __restrict__ q_pos,
                                                        const int32_t* __restrict__ kv_pos,
                                                        const int32_t* __restrict__ cu_q,
                                                        const int32_t* __restrict__ cu_kv,
                                                        int32_t* __restrict__ span) {
  __shared__ int32_t red[4];
  const int b = blockIdx.x;
  int32_t m = -1;
  for (int i = cu_kv[b] + threadIdx.x; i < cu_kv[b + 1]; i += 256) {
    const int32_t x = kv_pos[i];
    if (x != CP_POS_PAD_KV) m = max(m, x);
  }
  for (int i = cu_q[b] + threadIdx.x; i < cu_q[b + 1]; i += 256) m = max(m, q_pos[i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) span[b] = max(max(red[0], red[1]), max(red[2], red[3])) + 1;
}

// base[b] = exclusive prefix of span, saturating; one thread (batches are short lists)
__global__ void seq_base_kernel(const int32_t* __restrict__ span, int32_t batch,
                                int32_t* __restrict__ base) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int64_t acc = 0;
  for (int b = 0; b < batch; ++b) {
    base[b] = (int32_t)min<int64_t>(acc, INT32_MAX - 1);
    acc += span[b];
  }
}

// sequence of packed token i: last b with cu[b] <= i
__device__ __forceinline__ int seq_of(const int32_t* __restrict__ cu, int batch, int i) {
  int lo = 0, hi = batch;  // invariant: cu[lo] <= i < cu[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= i) lo = mid; else hi = mid;
  }
  return lo;
}

__global__ __launch_bounds__(256) void seq_encode_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ kv_pos,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv,
    const int32_t* __restrict__ base, int32_t batch, int32_t total_q, int32_t total_kv,
    int32_t* __restrict__ q_hi, int32_t* __restrict__ q_lo, int32_t* __restrict__ kv_enc) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < total_q) {
    const int32_t x = q_pos[i];
    const int64_t s = base[seq_of(cu_q, batch, i)];
    const bool ok = x >= 0 && s + x < INT32_MAX;
    q_hi[i] = ok ? (int32_t)(s + x) : CP_POS_PAD_Q;
    q_lo[i] = ok ? (int32_t)s : 0;
  }
  if (i < total_kv) {
    const int32_t x = kv_pos[i];
    const int64_t s = base[seq_of(cu_kv, batch, i)];
    kv_enc[i] = (x == CP_POS_PAD_KV || s + x >= INT32_MAX) ? CP_POS_PAD_KV : (int32_t)(s + x);
  }
}

}  // namespace

VarseqLayout varseq_layout(int32_t batch, int64_t total_q, int64_t total_kv) {
  VarseqLayout w;
  w.span_off = 0;
  w.base_off = round256((size_t)batch * 4);
  w.q_hi_off = w.base_off + round256((size_t)batch * 4);
  w.q_lo_off = w.q_hi_off + round256((size_t)total_q * 4);
  w.kv_off = w.q_lo_off + round256((size_t)total_q * 4);
  w.total = w.kv_off + round256((size_t)total_kv * 4);
  return w;
}

int launch_varseq_encode(int32_t batch, int64_t total_q, int64_t total_kv, const int32_t* q_pos,
                         const int32_t* kv_pos, const int32_t* cu_q, const int32_t* cu_kv,
                         void* workspace, hipStream_t stream) {
  const VarseqLayout w = varseq_layout(batch, total_q, total_kv);
  char* ws = (char*)workspace;
  int32_t* span = (int32_t*)(ws + w.span_off);
  int32_t* base = (int32_t*)(ws + w.base_off);
  hipLaunchKernelGGL(seq_span_kernel, dim3(batch), dim3(256), 0, stream, q_pos, kv_pos, cu_q,
                     cu_kv, span);
  hipLaunchKernelGGL(seq_base_kernel, dim3(1), dim3(64), 0, stream, span, batch, base);
  const int64_t n = std::max(total_q, total_kv);
  if (n > 0)
    hipLaunchKernelGGL(seq_encode_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       q_pos, kv_pos, cu_q, cu_kv, base, batch, (int32_t)total_q,
                       (int32_t)total_kv, (int32_t*)(ws + w.q_hi_off), (int32_t*)(ws + w.q_lo_off),
                       (int32_t*)(ws + w.kv_off));
  return check_launch();
}

}  // namespace cp
