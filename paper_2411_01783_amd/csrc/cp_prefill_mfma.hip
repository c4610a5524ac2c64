// bf16 MFMA partial attention for gfx950, head_dim 128: host side (launch plan, tile-bound
// pre-pass) and the definitions shared with the kernel in cp_prefill_pipe.h.
//
// Computes O, LSE = Attn(Q, KV) of one ring step (Algorithms 2 and 3; O and LSE as
// in Appendix B) for one KV head and its group of G = N_H / N_KV query heads.
//
// Work decomposition
//   - The (token, head-in-group) pairs of a KV head form R = total_q * G rows,
//     token-major. The causal mask depends on the token only, so all G heads of
//     a token share mask and K/V tile: GQA turns into a taller M dimension.
//   - A workgroup of 8 wavefronts owns 256 consecutive rows, 32 per wavefront,
//     and walks the KV axis in tiles of 128 keys brought straight into LDS
//     (double buffered), consumed in blocks of 32 keys by a three-stage software
//     pipeline per wavefront (see cp_prefill_pipe.h).
//   - Scores are produced transposed, S^T = K Q^T with v_mfma_f32_32x32x16_bf16:
//     a lane then holds 16 keys of ONE query per 32-key block, so the softmax
//     row statistics are per-lane scalars (one cross-lane exchange with lane^32)
//     and the exponentiated block is already in the B-operand layout of the
//     second product O^T += V^T P^T. No register shuffle between the products.
//   - Tile skipping (load-balanced sharding leaves half of every off-diagonal
//     step fully masked): a pre-pass records min/max kv_pos of every KV tile;
//     each workgroup compacts the tiles any of its queries can see into a list
//     in LDS and walks only those; only tiles that straddle a query position
//     pay for the mask.
//   - Short query shards (pass-Q partial prefill) are split over the KV axis
//     (grid.z); split results go to the workspace and are combined with Eq. 4.
//   - The epilogue transposes the accumulators through LDS so that every output
//     row leaves as one contiguous 512-byte (fp32) or 256-byte (bf16) run.
//   - Across ring steps the same body runs three ways: a launch per step into a stored
//     partial; a launch per step that merges into a running (O, LSE) in its epilogue
//     (ACC); or one launch per rank that walks the shards of all ring steps in ring
//     order, each behind an arrival flag, keeping the running softmax state in
//     registers (RING, prefill_ring_walk_kernel).
#include <type_traits>

#include "cp_common.h"

namespace cp {
namespace {

constexpr int D = 128;          // head_dim
constexpr int BM = 256;         // rows per workgroup
constexpr int TILE = 128;       // keys per LDS tile
constexpr int NWAVE = 8;        // wavefronts per workgroup
constexpr int NTHREADS = NWAVE * 64;
constexpr int POS_BYTES = TILE * 4;
constexpr int MAX_LIVE = 512;   // live-tile list entries per chunk (8 wavefronts x 64 tiles)
constexpr int OUT_STRIDE = D * 4 + 16;    // epilogue staging: one fp32 output row + pad
constexpr float kRescaleSlack = 8.f;               // log2 units
constexpr float kOverflowSum = 1099511627776.f;    // 2^40: a block sum beyond it is redone
constexpr float kDeadRowRef = 1e30f;               // reference of a row that sees no key
constexpr int kMinTilesPerSplit = 1;

struct Params {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  const int32_t* q_pos;
  const int32_t* kv_pos;
  const int32_t* q_lo;    // BAND only: smallest visible key position per query token
  const int2* bounds;     // [n_tiles] (min, max) of kv_pos per tile
  void* out;              // final output (n_splits == 1)
  float* lse;             // LSE output; ACC: the running LSE, read and written
  float* acc;             // ACC: running O, fp32 [rows_all_heads][D]
  void* final_out;        // ACC: where the merged O goes on the last step (else NULL)
  float* final_lse;       // ACC: optional copy of the merged LSE
  float* part_out;        // split scratch [n_splits][total_q * n_q_heads][D] fp32
  float* part_lse;        // [n_splits][total_q * n_q_heads]
  int64_t rows;           // R = total_q * G
  int64_t rows_all_heads; // total_q * n_q_heads
  int32_t group;          // G
  int32_t n_kv_heads;
  int32_t total_kv;
  int32_t n_tiles;
  int32_t tiles_per_split;
  int32_t n_splits;
  float scale_log2;       // softmax scale * log2(e)
};

// Ring walk in one launch (RING variant of prefill_mfma_kernel): the shards of a rank's ring
// steps, in ring order. Passed by value (kernel argument segment), so a step's entry is a
// scalar load with a uniform index.
constexpr int kMaxRingShards = 32;
struct RingShard {
  const bf16_t* k;
  const bf16_t* v;
  const int32_t* kv_pos;
  const int2* bounds;  // (min, max) of kv_pos per tile of this shard
  int32_t total_kv;    // tokens in this shard
  int32_t n_tiles;     // ceil(total_kv / TILE)
};
struct RingTable {
  RingShard shard[kMaxRingShards];
  const int32_t* arrived;  // or NULL: [n_shards], nonzero once the shard of step j may be read
  int32_t* error;          // bit j is set when the wait of step j gave up (only with `arrived`)
  int32_t n_shards;
  int32_t spin_limit;      // polls per shard before giving up
};
struct NoRing {};
template <bool RING>
using RingArg = typename std::conditional<RING, RingTable, NoRing>::type;

__global__ __launch_bounds__(256) void kv_tile_bounds_kernel(const int32_t* __restrict__ kv_pos,
                                                              int32_t total_kv, int32_t n_tiles,
                                                              int2* __restrict__ bounds) {
  const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tile >= n_tiles) return;
  const int lane = threadIdx.x & 63;
  int lo = INT32_MAX, hi = INT32_MIN;
#pragma unroll
  for (int h = 0; h < TILE / 64; ++h) {
    const int idx = tile * TILE + h * 64 + lane;
    if (idx < total_kv) {
      const int32_t x = kv_pos[idx];
      lo = min(lo, x);
      hi = max(hi, x);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = min(lo, __shfl_xor(lo, o, 64));
    hi = max(hi, __shfl_xor(hi, o, 64));
  }
  if (lane == 0) bounds[tile] = make_int2(lo, hi);
}

// The same for the shards of a whole ring in one launch (a launch per shard costs more than
// the work: a shard of 8K keys is 64 tiles).
struct BoundsTable {
  const int32_t* kv_pos[CP_MAX_PARTS];
  int2* bounds[CP_MAX_PARTS];
  int32_t total_kv[CP_MAX_PARTS];
  int32_t tile_begin[CP_MAX_PARTS + 1];  // first global tile index of every shard
  int32_t n_shards;
};
__global__ __launch_bounds__(256) void kv_tile_bounds_ring_kernel(const BoundsTable t) {
  const int gt = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (gt >= t.tile_begin[t.n_shards]) return;
  int j = 0;
  while (t.tile_begin[j + 1] <= gt) ++j;  // (wave-uniform; empty shards are skipped over)
  const int tile = gt - t.tile_begin[j];
  const int32_t* __restrict__ kv_pos = t.kv_pos[j];
  const int32_t total_kv = t.total_kv[j];
  const int lane = threadIdx.x & 63;
  int lo = INT32_MAX, hi = INT32_MIN;
#pragma unroll
  for (int h = 0; h < TILE / 64; ++h) {
    const int idx = tile * TILE + h * 64 + lane;
    if (idx < total_kv) {
      const int32_t x = kv_pos[idx];
      lo = min(lo, x);
      hi = max(hi, x);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = min(lo, __shfl_xor(lo, o, 64));
    hi = max(hi, __shfl_xor(hi, o, 64));
  }
  if (lane == 0) t.bounds[j][tile] = make_int2(lo, hi);
}

__device__ __forceinline__ floatx16_t mfma32(bf16x8_t a, bf16x8_t b, floatx16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Value of lane ^ 32 (v_permlane32_swap: no LDS round trip).
__device__ __forceinline__ float xor32(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

#include "cp_prefill_pipe.h"

struct Plan {
  int n_tiles, n_row_blocks, n_splits, tiles_per_split;
  size_t bounds_bytes, part_out_bytes, part_lse_bytes;
};

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// `merging`: the call merges into a running result in its epilogue, which only unsplit
// launches do; then (and for the ring walk) the KV axis is left whole from 128 workgroups on.
Plan make_plan(const cp_shape& s, bool merging = false) {
  Plan pl;
  const int group = s.n_q_heads / s.n_kv_heads;
  const int64_t rows = s.total_q * group;
  pl.n_tiles = (int)((s.total_kv + TILE - 1) / TILE);
  pl.n_row_blocks = (int)((rows + BM - 1) / BM);
  // Split the KV axis when the row blocks alone cannot occupy the 256 CUs (the cost model
  // below keeps 129 .. 255 workgroups whole: two splits would need a second round). Every split
  // costs one fp32 partial of the output, so keep at least kMinTilesPerSplit tiles per split.
  const int64_t wgs = (int64_t)pl.n_row_blocks * s.n_kv_heads;
  int splits = 1;
  if (wgs > 0 && wgs < (merging ? 128 : 256) && pl.n_tiles >= 2 * kMinTilesPerSplit) {
    // Cost of a split count, in units of one tile step of a workgroup: the workgroups run in
    // rounds of 256 (one per CU), each round walks its tiles plus about three tile steps of
    // start-up and epilogue, and every split adds one fp32 partial to write and to merge.
    const int max_splits = (int)std::min<int64_t>(pl.n_tiles / kMinTilesPerSplit, CP_MAX_PARTS);
    const double partial_cost = (double)s.total_q * s.n_q_heads * 4.8e-5;
    double best = 0.0;
    for (int c = 1; c <= max_splits; ++c) {
      const int tps = (pl.n_tiles + c - 1) / c;
      const int ns = (pl.n_tiles + tps - 1) / tps;
      if (ns != c) continue;  // the same split as a smaller count
      const int64_t rounds = (wgs * ns + 255) / 256;
      const double cost = (double)rounds * (tps + 3) + partial_cost * ns;
      if (splits == 1 && c == 1) best = cost;
      if (cost < best) {
        best = cost;
        splits = c;
      }
    }
  }
  pl.tiles_per_split = pl.n_tiles > 0 ? (pl.n_tiles + splits - 1) / splits : 1;
  pl.n_splits = pl.n_tiles > 0 ? (pl.n_tiles + pl.tiles_per_split - 1) / pl.tiles_per_split : 1;
  pl.bounds_bytes = round256((size_t)std::max(pl.n_tiles, 1) * sizeof(int2));
  const size_t rows_all = (size_t)s.total_q * s.n_q_heads;
  pl.part_out_bytes = pl.n_splits > 1 ? round256((size_t)pl.n_splits * rows_all * D * 4) : 0;
  pl.part_lse_bytes = pl.n_splits > 1 ? round256((size_t)pl.n_splits * rows_all * 4) : 0;
  return pl;
}

}  // namespace

size_t prefill_mfma_workspace_bytes(const cp_shape& s) {
  const Plan pl = make_plan(s);
  return pl.bounds_bytes + pl.part_out_bytes + pl.part_lse_bytes;
}

size_t kv_tile_bounds_bytes(int64_t total_kv) {
  return round256((size_t)std::max<int64_t>((total_kv + TILE - 1) / TILE, 1) * sizeof(int2));
}

int launch_kv_tile_bounds(const int32_t* kv_pos, int64_t total_kv, void* bounds_out,
                          hipStream_t stream) {
  const int n_tiles = (int)((total_kv + TILE - 1) / TILE);
  if (n_tiles == 0) return CP_OK;
  hipLaunchKernelGGL(kv_tile_bounds_kernel, dim3((n_tiles + 3) / 4), dim3(256), 0, stream, kv_pos,
                     (int32_t)total_kv, n_tiles, (int2*)bounds_out);
  return check_launch();
}

int launch_kv_tile_bounds_ring(int n_shards, const int32_t* const* kv_pos, const int64_t* n_kv,
                               void* const* bounds_out, hipStream_t stream) {
  if (n_shards < 1 || n_shards > CP_MAX_PARTS) return CP_ERR_SHAPE;
  BoundsTable t = {};
  int64_t tiles = 0;
  for (int j = 0; j < n_shards; ++j) {
    if (n_kv[j] < 0 || n_kv[j] > INT32_MAX - TILE) return CP_ERR_SHAPE;
    if (n_kv[j] > 0 && (kv_pos[j] == nullptr || bounds_out[j] == nullptr)) return CP_ERR_NULL;
    t.kv_pos[j] = kv_pos[j];
    t.bounds[j] = (int2*)bounds_out[j];
    t.total_kv[j] = (int32_t)n_kv[j];
    t.tile_begin[j] = (int32_t)tiles;
    tiles += (n_kv[j] + TILE - 1) / TILE;
    if (tiles > INT32_MAX - 4) return CP_ERR_SHAPE;
  }
  t.tile_begin[n_shards] = (int32_t)tiles;
  t.n_shards = n_shards;
  if (tiles == 0) return CP_OK;
  hipLaunchKernelGGL(kv_tile_bounds_ring_kernel, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0,
                     stream, t);
  return check_launch();
}

bool prefill_mfma_splits_kv(const cp_shape& s, bool merging) {
  return make_plan(s, merging).n_splits > 1;
}

int launch_prefill_mfma(const cp_shape& s, float scale, const void* q, const void* k,
                        const void* v, const int32_t* q_pos, const int32_t* kv_pos, void* out,
                        float* lse, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                        const void* tile_bounds, const int32_t* q_lo, hipStream_t stream,
                        const PrefillAccumulate* acc) {
  const Plan pl = make_plan(s, acc != nullptr);
  if (acc != nullptr && (pl.n_splits > 1 || q_lo != nullptr)) return CP_ERR_UNSUPPORTED;
  if (workspace_bytes < pl.bounds_bytes + pl.part_out_bytes + pl.part_lse_bytes)
    return CP_ERR_WORKSPACE;
  if (pl.n_row_blocks == 0) return CP_OK;
  if (s.n_kv_heads > 65535 || pl.n_splits > 65535) return CP_ERR_SHAPE;
  if (s.total_q * (s.n_q_heads / s.n_kv_heads) > 0x7fffffffLL) return CP_ERR_SHAPE;  // 31-bit rows

  char* ws = (char*)workspace;
  Params p;
  p.q = (const bf16_t*)q; p.k = (const bf16_t*)k; p.v = (const bf16_t*)v;
  p.q_pos = q_pos; p.kv_pos = kv_pos; p.q_lo = q_lo;
  p.bounds = tile_bounds != nullptr ? (const int2*)tile_bounds : (const int2*)ws;
  p.out = out; p.lse = lse;
  p.acc = nullptr; p.final_out = nullptr; p.final_lse = nullptr;
  if (acc != nullptr) {
    p.out = nullptr; p.lse = acc->lse; p.acc = acc->out;
    p.final_out = acc->final_out; p.final_lse = acc->final_lse;
  }
  p.part_out = (float*)(ws + pl.bounds_bytes);
  p.part_lse = (float*)(ws + pl.bounds_bytes + pl.part_out_bytes);
  p.group = s.n_q_heads / s.n_kv_heads;
  p.rows = s.total_q * p.group;
  p.rows_all_heads = s.total_q * s.n_q_heads;
  p.n_kv_heads = s.n_kv_heads;
  p.total_kv = (int32_t)s.total_kv;
  p.n_tiles = pl.n_tiles;
  p.tiles_per_split = pl.tiles_per_split;
  p.n_splits = pl.n_splits;
  p.scale_log2 = scale * kLog2e;

  if (tile_bounds == nullptr && launch_kv_tile_bounds(kv_pos, s.total_kv, ws, stream) != CP_OK)
    return CP_ERR_LAUNCH;

  const dim3 grid(pl.n_row_blocks, s.n_kv_heads, pl.n_splits);
  const bool direct_bf16 = pl.n_splits == 1 && out_dtype == CP_BF16;
  const bool band = q_lo != nullptr;
  auto kern = acc != nullptr
                  ? (acc->final_out != nullptr && acc->final_dtype == CP_BF16
                         ? prefill_mfma_kernel<bf16_t, false, false, true>
                         : prefill_mfma_kernel<float, false, false, true>)
              : pl.n_splits > 1
                  ? (band ? prefill_mfma_kernel<float, true, true> : prefill_mfma_kernel<float, false, true>)
                  : direct_bf16
                        ? (band ? prefill_mfma_kernel<bf16_t, true, false>
                                : prefill_mfma_kernel<bf16_t, false, false>)
                        : (band ? prefill_mfma_kernel<float, true, false>
                                : prefill_mfma_kernel<float, false, false>);
  constexpr int kSmem = SMEM_BYTES8;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                          kSmem) != hipSuccess)
    return CP_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), kSmem, stream, p, p.bounds);
  if (check_launch() != CP_OK) return CP_ERR_LAUNCH;

  if (pl.n_splits > 1)
    return launch_merge_strided(p.rows_all_heads, D, pl.n_splits, p.part_out, p.part_lse,
                                p.rows_all_heads, out, out_dtype, lse, stream);
  return CP_OK;
}

bool prefill_ring_walk_applies(const cp_shape& s, int n_shards) {
  if (n_shards < 1 || n_shards > kMaxRingShards) return false;
  const Plan pl = make_plan(s, true);
  return pl.n_row_blocks > 0 && pl.n_splits == 1;
}

int launch_prefill_mfma_ring(const cp_shape& s, float scale, const void* q, const int32_t* q_pos,
                             int n_shards, const void* const* k, const void* const* v,
                             const int32_t* const* kv_pos, const void* const* bounds,
                             const int64_t* n_kv, const int32_t* arrived, int32_t* error,
                             int32_t spin_limit, void* out, float* lse, int32_t out_dtype,
                             hipStream_t stream) {
  if (!prefill_ring_walk_applies(s, n_shards)) return CP_ERR_UNSUPPORTED;
  if (arrived != nullptr && (error == nullptr || spin_limit < 1)) return CP_ERR_SHAPE;
  if (s.n_kv_heads > 65535) return CP_ERR_SHAPE;
  if (s.total_q * (s.n_q_heads / s.n_kv_heads) > 0x7fffffffLL) return CP_ERR_SHAPE;  // 31-bit rows
  const Plan pl = make_plan(s, true);
  Params p = {};
  p.q = (const bf16_t*)q; p.q_pos = q_pos;
  p.k = (const bf16_t*)k[0]; p.v = (const bf16_t*)v[0]; p.kv_pos = kv_pos[0];
  p.bounds = (const int2*)bounds[0];
  p.out = out; p.lse = lse;
  p.group = s.n_q_heads / s.n_kv_heads;
  p.rows = s.total_q * p.group;
  p.rows_all_heads = s.total_q * s.n_q_heads;
  p.n_kv_heads = s.n_kv_heads;
  p.total_kv = (int32_t)s.total_kv;
  p.n_tiles = pl.n_tiles;
  p.tiles_per_split = pl.tiles_per_split;
  p.n_splits = 1;
  p.scale_log2 = scale * kLog2e;
  RingTable rt = {};
  for (int j = 0; j < n_shards; ++j) {
    if (n_kv[j] < 0 || n_kv[j] > INT32_MAX - TILE) return CP_ERR_SHAPE;
    if (n_kv[j] > 0 &&
        (k[j] == nullptr || v[j] == nullptr || kv_pos[j] == nullptr || bounds[j] == nullptr))
      return CP_ERR_NULL;
    rt.shard[j].total_kv = (int32_t)n_kv[j];
    rt.shard[j].n_tiles = (int32_t)((n_kv[j] + TILE - 1) / TILE);
    rt.shard[j].k = (const bf16_t*)k[j];
    rt.shard[j].v = (const bf16_t*)v[j];
    rt.shard[j].kv_pos = kv_pos[j];
    rt.shard[j].bounds = (const int2*)bounds[j];
  }
  rt.arrived = arrived; rt.error = error; rt.n_shards = n_shards; rt.spin_limit = spin_limit;
  auto kern = out_dtype == CP_BF16 ? prefill_ring_walk_kernel<bf16_t>
                                   : prefill_ring_walk_kernel<float>;
  constexpr int kSmem = SMEM_BYTES8;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                          kSmem) != hipSuccess)
    return CP_ERR_LAUNCH;
  const dim3 grid(pl.n_row_blocks, s.n_kv_heads, 1);
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), kSmem, stream, p, rt);
  return check_launch();
}

}  // namespace cp

