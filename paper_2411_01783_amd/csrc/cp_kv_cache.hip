// One rank's share of the persistent KV cache (Sections 3.5.2 and 3.6): the K/V of every
// turn's new tokens, decode tokens included, are appended to the share of the rank that owns
// them and stay there for later turns.
//
// Layout: packed [slots, n_kv_heads, head_dim] with sequence b owning the slot range
// [cu_kv[b], cu_kv[b+1]) (its capacity on this rank). The first used[b] slots hold tokens, in
// the order they arrived; every other slot carries CP_POS_PAD_KV in the position array, which
// no query position can reach, so the attention kernels read the cache as it is.
//
// Pure data movement, HBM-bound: one 16-byte chunk of K and of V per thread.
#include "cp_common.h"

namespace cp {
namespace {

struct AppendParams {
  const uint4* k_new;
  const uint4* v_new;
  const int32_t* pos_new;
  const int32_t* cu_new;
  uint4* k_cache;
  uint4* v_cache;
  int32_t* pos_cache;
  const int32_t* cu_kv;
  int32_t* used;
  int32_t* dropped;
  int32_t batch;
  int32_t chunks_per_token;  // 16-byte chunks in one token's K (or V) row
  int64_t n_new;
  int64_t slots;
};

constexpr int64_t kTicketMaxBlocks = 64;  // above: two launches, see kv_append_kernel

// Sequence that new token i belongs to: the b with cu_new[b] <= i < cu_new[b+1].
__device__ __forceinline__ int find_sequence(const int32_t* cu_new, int batch, int64_t i) {
  int lo = 0, hi = batch;  // invariant: cu_new[lo] <= i < cu_new[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_new[mid] <= i) lo = mid; else hi = mid;
  }
  return lo;
}

// seq_used[] may only change once every workgroup has read it.
// TICKET (calls of a few workgroups, e.g. a decode step's tokens): one launch. Every workgroup
// takes a ticket (the word after the last sequence's count) after its reads; the one that
// draws the last ticket advances the counts, counts what did not fit and zeroes the ticket
// word. Tickets are atomics on one address, about 10 ns each across XCDs, so large calls use
// a second launch (kv_append_commit_kernel) instead.
__device__ __forceinline__ void commit_counts(const AppendParams& p) {
  for (int b = threadIdx.x; b < p.batch; b += blockDim.x) {
    const int32_t n_new = p.cu_new[b + 1] - p.cu_new[b];
    const int32_t room = p.cu_kv[b + 1] - p.cu_kv[b] - p.used[b];
    int32_t taken = n_new < room ? n_new : room;
    if (taken < 0) taken = 0;
    p.used[b] += taken;
    if (p.dropped != nullptr && n_new > taken) atomicAdd(p.dropped, n_new - taken);
  }
}

template <bool TICKET>
__global__ __launch_bounds__(256) void kv_append_kernel(AppendParams p) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t i = t / p.chunks_per_token;
  if (i < p.n_new) {
    const int c = (int)(t - i * p.chunks_per_token);
    const int b = find_sequence(p.cu_new, p.batch, i);
    const int64_t first = p.cu_kv[b], used = p.used[b], off = i - p.cu_new[b];
    const int64_t slot = first + used + off;
    // Over capacity: dropped (counted at the commit). The remaining conditions hold for
    // consistent bookkeeping arrays; they keep inconsistent ones from writing outside the cache.
    if (slot < p.cu_kv[b + 1] && slot < p.slots && first >= 0 && used >= 0 && off >= 0) {
      const int64_t src = i * p.chunks_per_token + c;
      const int64_t dst = slot * p.chunks_per_token + c;
      p.k_cache[dst] = p.k_new[src];
      p.v_cache[dst] = p.v_new[src];
      if (c == 0) p.pos_cache[slot] = p.pos_new[i];
    }
  }
  if (!TICKET) return;
  __shared__ int last;
  __syncthreads();  // every thread of the workgroup has read its count
  // No fence: what must come first are the workgroups' *reads* of the counts, and those have
  // returned their values before the barrier above. (A release fence here would write back
  // the L2 of the workgroup's XCD, K/V rows included, once per workgroup.)
  if (threadIdx.x == 0) last = atomicAdd(p.used + p.batch, 1) == (int)gridDim.x - 1;
  __syncthreads();
  if (!last) return;
  commit_counts(p);
  if (threadIdx.x == 0) p.used[p.batch] = 0;
}

// Second launch of a large call, after kv_append_kernel<false> on the same stream.
__global__ __launch_bounds__(256) void kv_append_commit_kernel(AppendParams p) {
  commit_counts(p);
}

// Unused slots must not hold NaN or Inf patterns: a masked key still enters the P V product
// with weight zero. So a reset clears K and V as well as the bookkeeping.
__global__ __launch_bounds__(256) void kv_cache_reset_kernel(uint4* k_cache, uint4* v_cache,
                                                             int64_t chunks, int32_t* pos_cache,
                                                             int64_t slots, int32_t* used,
                                                             int32_t batch, int32_t* dropped) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
  for (int64_t c = t; c < chunks; c += stride) {
    k_cache[c] = zero;
    v_cache[c] = zero;
  }
  for (int64_t i = t; i < slots; i += stride) pos_cache[i] = CP_POS_PAD_KV;
  for (int64_t i = t; i <= batch; i += stride) used[i] = 0;  // counts and the ticket word
  if (t == 0 && dropped != nullptr) *dropped = 0;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace
}  // namespace cp

extern "C" {

int cp_kv_cache_reset(const cp_shape* shape, void* k_cache, void* v_cache,
                      int32_t* kv_pos_cache, int32_t* seq_used, int32_t* dropped, void* stream) {
  if (shape == nullptr) return CP_ERR_NULL;
  const cp_shape& s = *shape;
  if (s.dtype != CP_BF16 && s.dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if (s.head_dim < 8 || s.head_dim > 256 || s.head_dim % 8 != 0) return CP_ERR_UNSUPPORTED;
  if (s.n_kv_heads < 1 || s.batch < 1 || s.total_kv < 0 || s.total_kv > INT32_MAX)
    return CP_ERR_SHAPE;
  if (seq_used == nullptr) return CP_ERR_NULL;
  if (s.total_kv > 0 && (k_cache == nullptr || v_cache == nullptr || kv_pos_cache == nullptr))
    return CP_ERR_NULL;
  if (!cp::aligned16(k_cache) || !cp::aligned16(v_cache)) return CP_ERR_ALIGN;
  const int64_t row_bytes = (int64_t)s.n_kv_heads * s.head_dim * (s.dtype == CP_BF16 ? 2 : 4);
  const int64_t chunks = s.total_kv * (row_bytes / 16);
  int64_t work = chunks > s.batch ? chunks : s.batch;
  int64_t blocks = (work + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;  // grid-stride beyond that
  hipLaunchKernelGGL(cp::kv_cache_reset_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     (hipStream_t)stream, (uint4*)k_cache, (uint4*)v_cache, chunks, kv_pos_cache,
                     s.total_kv, seq_used, s.batch, dropped);
  return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
}

int cp_kv_append(const cp_shape* shape, const void* k_new, const void* v_new,
                 const int32_t* pos_new, const int32_t* cu_seqlens_new, void* k_cache,
                 void* v_cache, int32_t* kv_pos_cache, const int32_t* cu_seqlens_kv,
                 int32_t* seq_used, int32_t* dropped, void* stream) {
  if (shape == nullptr) return CP_ERR_NULL;
  const cp_shape& s = *shape;
  if (s.dtype != CP_BF16 && s.dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if (s.head_dim < 8 || s.head_dim > 256 || s.head_dim % 8 != 0) return CP_ERR_UNSUPPORTED;
  if (s.n_kv_heads < 1 || s.batch < 1 || s.total_q < 0 || s.total_kv < 0) return CP_ERR_SHAPE;
  if (s.total_kv > INT32_MAX || s.total_q > INT32_MAX) return CP_ERR_SHAPE;
  if (cu_seqlens_new == nullptr || cu_seqlens_kv == nullptr || seq_used == nullptr)
    return CP_ERR_NULL;
  if (s.total_q == 0) return CP_OK;
  if (k_new == nullptr || v_new == nullptr || pos_new == nullptr || k_cache == nullptr ||
      v_cache == nullptr || kv_pos_cache == nullptr)
    return CP_ERR_NULL;
  if (!cp::aligned16(k_new) || !cp::aligned16(v_new) || !cp::aligned16(k_cache) ||
      !cp::aligned16(v_cache))
    return CP_ERR_ALIGN;
  const int64_t row_bytes = (int64_t)s.n_kv_heads * s.head_dim * (s.dtype == CP_BF16 ? 2 : 4);
  cp::AppendParams p;
  p.k_new = (const uint4*)k_new; p.v_new = (const uint4*)v_new;
  p.pos_new = pos_new; p.cu_new = cu_seqlens_new;
  p.k_cache = (uint4*)k_cache; p.v_cache = (uint4*)v_cache; p.pos_cache = kv_pos_cache;
  p.cu_kv = cu_seqlens_kv; p.used = seq_used; p.dropped = dropped;
  p.batch = s.batch; p.chunks_per_token = (int32_t)(row_bytes / 16); p.n_new = s.total_q;
  p.slots = s.total_kv;
  const int64_t threads = s.total_q * p.chunks_per_token;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > INT32_MAX) return CP_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  if (blocks <= cp::kTicketMaxBlocks) {
    hipLaunchKernelGGL(cp::kv_append_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(cp::kv_append_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, p);
  if (hipGetLastError() != hipSuccess) return CP_ERR_LAUNCH;
  hipLaunchKernelGGL(cp::kv_append_commit_kernel, dim3(1), dim3(256), 0, st, p);
  return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
}

int32_t cp_decode_owner(int32_t seq, int32_t decode_iter, int32_t n_ranks) {
  if (n_ranks < 1 || seq < 0 || decode_iter < 0) return CP_ERR_SHAPE;
  return (int32_t)(((int64_t)seq + decode_iter) % n_ranks);
}

}  // extern "C"
