// Internal declarations shared by the HIP translation units of libcp_attn.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cp_attn.h"

namespace cp {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return static_cast<float>(x); }

template <typename T>
__device__ __forceinline__ T from_float(float x);
template <>
__device__ __forceinline__ float from_float<float>(float x) {
  return x;
}
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float x) {
  return static_cast<bf16_t>(x);
}

// ---- launchers (each returns a cp_status; enqueue on `stream` only) ----

// fp32 vector kernel: any supported dtype / head_dim, packed batches.
int launch_partial_generic(const cp_shape& s, float scale, const void* q, const void* k,
                           const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                           const int32_t* cu_q, const int32_t* cu_kv, void* out, float* lse,
                           int32_t out_dtype, hipStream_t stream);

// bf16 MFMA kernel, head_dim 128, batch 1.
// `tile_bounds`, when not NULL, holds the per-tile (min, max) of kv_pos already computed by
// launch_kv_tile_bounds for this kv_pos array; otherwise the launcher computes it into the
// workspace first.
size_t prefill_mfma_workspace_bytes(const cp_shape& s);
size_t kv_tile_bounds_bytes(int64_t total_kv);
int launch_kv_tile_bounds(const int32_t* kv_pos, int64_t total_kv, void* bounds_out,
                          hipStream_t stream);
// Tile bounds of all shards of a ring in one launch; bounds_out[j] as for launch_kv_tile_bounds.
int launch_kv_tile_bounds_ring(int n_shards, const int32_t* const* kv_pos, const int64_t* n_kv,
                               void* const* bounds_out, hipStream_t stream);
// `acc`, when not NULL, turns the launch into "merge into a running result": out / lse /
// out_dtype are ignored, (acc->out, acc->lse) are read and updated (Equation 4), and if
// acc->final_out is not NULL the merged O goes there in acc->final_dtype instead of back to
// acc->out. Only for launches that do not split the KV axis and are not packed batches.
struct PrefillAccumulate {
  float* out;        // fp32 [total_q, n_q_heads, head_dim]
  float* lse;        // fp32 [total_q, n_q_heads]
  void* final_out;   // or NULL
  float* final_lse;  // or NULL
  int32_t final_dtype;
};
// `merging`: for a call that merges into a running result in its epilogue (see make_plan).
bool prefill_mfma_splits_kv(const cp_shape& s, bool merging);
int launch_prefill_mfma(const cp_shape& s, float scale, const void* q, const void* k,
                        const void* v, const int32_t* q_pos, const int32_t* kv_pos, void* out,
                        float* lse, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                        const void* tile_bounds, const int32_t* q_lo, hipStream_t stream,
                        const PrefillAccumulate* acc = nullptr);

// One launch for all ring steps of a rank (pass-KV): the shards k[j], v[j], kv_pos[j] (n_kv[j]
// tokens each; any sizes, empty ones included) with their tile bounds, in ring order
// j = 0..n_shards-1, walked by every workgroup with one running softmax state; writes the
// rank's merged O / LSE. s.total_kv is the largest shard (it decides, with total_q, whether
// the launch would split its KV axis, which the walk does not support).
// `arrived` (device, or NULL): int32 per step, the kernel waits (at most spin_limit polls) for
// a nonzero value before it reads step j's shard; a wait that gives up sets bit j of *error
// and leaves the shard out.
bool prefill_ring_walk_applies(const cp_shape& s, int n_shards);
int launch_prefill_mfma_ring(const cp_shape& s, float scale, const void* q, const int32_t* q_pos,
                             int n_shards, const void* const* k, const void* const* v,
                             const int32_t* const* kv_pos, const void* const* bounds,
                             const int64_t* n_kv, const int32_t* arrived, int32_t* error,
                             int32_t spin_limit, void* out, float* lse, int32_t out_dtype,
                             hipStream_t stream);

// Packed batches on the MFMA path: per-sequence position ranges (see cp_varseq.hip).
struct VarseqLayout {
  size_t span_off, base_off, q_hi_off, q_lo_off, kv_off, total;
};
VarseqLayout varseq_layout(int32_t batch, int64_t total_q, int64_t total_kv);
int launch_varseq_encode(int32_t batch, int64_t total_q, int64_t total_kv, const int32_t* q_pos,
                         const int32_t* kv_pos, const int32_t* cu_q, const int32_t* cu_kv,
                         void* workspace, hipStream_t stream);

// split-KV decode, bf16, head_dim 128.
size_t decode_workspace_bytes(const cp_shape& s);
int launch_decode(const cp_shape& s, float scale, const void* q, const void* k, const void* v,
                  const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_kv,
                  const int32_t* bid, void* out, float* lse, int32_t out_dtype, void* workspace,
                  size_t workspace_bytes, hipStream_t stream);

// Flat split-KV decode (cp_shape.flags has CP_SHAPE_UNIQUE_BID): the partials of one KV holder
// go to `region` (decode_flat_region_bytes), and one merge launch applies Equation 4 over the
// regions of n_holders holders (shapes[k], regions[k], cu_kv[k] describe holder k; all share
// the queries' bid, n_q and head counts).
bool decode_flat_applies(const cp_shape& s);
size_t decode_flat_region_bytes(const cp_shape& s);
int launch_decode_flat_partials(const cp_shape& s, float scale, const void* q, const void* k,
                                const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                                const int32_t* cu_kv, const int32_t* bid, void* region,
                                size_t region_bytes, hipStream_t stream);
int launch_decode_flat_merge(int n_holders, const cp_shape* shapes, void* const* regions,
                             const int32_t* const* cu_kv, const int32_t* bid, int64_t n_q,
                             void* out, int32_t out_dtype, float* lse, hipStream_t stream);

// Equation 4 over n_parts partials given as device pointers.
int launch_merge(int64_t rows, int32_t head_dim, int32_t n_parts, const void* const* outs,
                 const float* const* lses, int32_t part_dtype, void* out, int32_t out_dtype,
                 float* lse_out, hipStream_t stream);

// Equation 4 over n_parts partials laid out with a constant stride (split-KV scratch).
int launch_merge_strided(int64_t rows, int32_t head_dim, int32_t n_parts, const float* parts_out,
                         const float* parts_lse, int64_t part_stride_rows, void* out,
                         int32_t out_dtype, float* lse_out, hipStream_t stream);

inline int check_launch() {
  return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
}

}  // namespace cp
