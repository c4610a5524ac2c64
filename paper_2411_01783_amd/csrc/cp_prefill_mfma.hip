// bf16 MFMA partial attention for gfx950, head_dim 128.
//
// Computes O, LSE = Attn(Q, KV) of one ring step (Algorithms 2 and 3; O and LSE as
// in Appendix B) for one KV head and its group of G = N_H / N_KV query heads.
//
// Work decomposition
//   - The (token, head-in-group) pairs of a KV head form R = total_q * G rows,
//     token-major. The causal mask depends on the token only, so all G heads of
//     a token share mask and K/V tile: GQA turns into a taller M dimension.
//   - A workgroup of 8 wavefronts owns 256 consecutive rows, 32 per wavefront,
//     and walks the KV axis in tiles of 64 keys staged through LDS (double
//     buffered; K as [key][d], V transposed to [d][key] while it is stored).
//   - Scores are produced transposed, S^T = K Q^T with v_mfma_f32_32x32x16_bf16:
//     a lane then holds 16 keys of ONE query per 32-key block, so the softmax
//     row statistics are per-lane scalars (one cross-lane exchange with lane^32)
//     and the exponentiated block is already in the B-operand layout of the
//     second product O^T += V^T P^T. No register shuffle between the products.
//   - Tile skipping (load-balanced sharding leaves half of every off-diagonal
//     step fully masked): a pre-pass records min/max kv_pos of every KV tile;
//     a workgroup skips tiles whose smallest position exceeds its largest query
//     position, and only tiles that straddle a query position pay for the mask.
//   - Short query shards (pass-Q partial prefill) are split over the KV axis
//     (grid.z); split results go to the workspace and are combined with Eq. 4.
#include "cp_common.h"

namespace cp {
namespace {

constexpr int D = 128;         // head_dim
constexpr int BM = 256;        // rows per workgroup
constexpr int BN = 64;         // keys per tile
constexpr int NWAVE = 8;       // wavefronts per workgroup
constexpr int NTHREADS = NWAVE * 64;
constexpr int K_STRIDE = D * 2 + 16;   // bytes per key row in LDS (+16: conflict-free b128 reads)
constexpr int VT_STRIDE = BN * 2 + 16; // bytes per d row of transposed V
constexpr int K_BYTES = BN * K_STRIDE;
constexpr int VT_BYTES = D * VT_STRIDE;
constexpr int SMEM_BYTES = 2 * K_BYTES + 2 * VT_BYTES + 64;

struct Params {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  const int32_t* q_pos;
  const int32_t* kv_pos;
  const int2* bounds;     // [n_tiles] (min, max) of kv_pos per tile
  void* out;              // final output (n_splits == 1)
  float* lse;
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

__global__ __launch_bounds__(256) void kv_tile_bounds_kernel(const int32_t* __restrict__ kv_pos,
                                                              int32_t total_kv, int32_t n_tiles,
                                                              int2* __restrict__ bounds) {
  const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tile >= n_tiles) return;
  const int lane = threadIdx.x & 63;
  const int idx = tile * BN + lane;
  int lo = INT32_MAX, hi = INT32_MIN;
  if (idx < total_kv) lo = hi = kv_pos[idx];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = min(lo, __shfl_xor(lo, o, 64));
    hi = max(hi, __shfl_xor(hi, o, 64));
  }
  if (lane == 0) bounds[tile] = make_int2(lo, hi);
}

__device__ __forceinline__ floatx16_t mfma32(bf16x8_t a, bf16x8_t b, floatx16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// Global -> register staging of one KV tile (held across the compute of the previous tile).
struct TileRegs {
  uint4 k[2];  // 2 x 8 bf16 of K
  uint2 v[4];  // 4 keys x 4 bf16 of V
};

__device__ __forceinline__ void load_tile(const Params& p, int kvh, int tile, int tid,
                                          TileRegs& r) {
  const int key0 = tile * BN;
  const int64_t head_off = (int64_t)kvh * D;
  const int64_t tok_stride = (int64_t)p.n_kv_heads * D;
#pragma unroll
  for (int pp = 0; pp < 2; ++pp) {
    const int key = key0 + pp * 32 + (tid >> 4);
    r.k[pp] = make_uint4(0, 0, 0, 0);
    if (key < p.total_kv)
      r.k[pp] = *(const uint4*)(p.k + key * tok_stride + head_off + (tid & 15) * 8);
  }
  const int kq = tid >> 5, dc = tid & 31;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int key = key0 + kq * 4 + b;
    r.v[b] = make_uint2(0, 0);
    if (key < p.total_kv) r.v[b] = *(const uint2*)(p.v + key * tok_stride + head_off + dc * 4);
  }
}

// Register -> LDS. K keeps its [key][d] layout. V is transposed: physical row
// rho = (d % 4) * 32 + d / 4 holds channel d, and inside every block of 16 keys the key
// (a*8 + g*4 + b) sits at slot (g*8 + a*4 + b), which is the order in which the
// accumulator of S^T hands the probabilities to the second product.
__device__ __forceinline__ void store_tile(char* kbuf, char* vtbuf, int tid, const TileRegs& r) {
#pragma unroll
  for (int pp = 0; pp < 2; ++pp)
    *(uint4*)(kbuf + (pp * 32 + (tid >> 4)) * K_STRIDE + (tid & 15) * 16) = r.k[pp];
  const int kq = tid >> 5, dc = tid & 31;
  const int blk = kq >> 2, a = (kq & 3) >> 1, g = kq & 1;
  const int slot0 = blk * 16 + g * 8 + a * 4;
  const uint32_t x0 = r.v[0].x, x1 = r.v[1].x, x2 = r.v[2].x, x3 = r.v[3].x;
  const uint32_t y0 = r.v[0].y, y1 = r.v[1].y, y2 = r.v[2].y, y3 = r.v[3].y;
  uint2 t[4];
  t[0] = make_uint2((x0 & 0xffffu) | (x1 << 16), (x2 & 0xffffu) | (x3 << 16));
  t[1] = make_uint2((x0 >> 16) | (x1 & 0xffff0000u), (x2 >> 16) | (x3 & 0xffff0000u));
  t[2] = make_uint2((y0 & 0xffffu) | (y1 << 16), (y2 & 0xffffu) | (y3 << 16));
  t[3] = make_uint2((y0 >> 16) | (y1 & 0xffff0000u), (y2 >> 16) | (y3 & 0xffff0000u));
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *(uint2*)(vtbuf + (i * 32 + dc) * VT_STRIDE + slot0 * 2) = t[i];
}

template <typename TO>
__global__ __launch_bounds__(NTHREADS) void prefill_mfma_kernel(Params p) {
  extern __shared__ __align__(16) char smem[];
  char* const kbuf0 = smem;
  char* const vtbuf0 = smem + 2 * K_BYTES;
  int* const wg_minmax = (int*)(smem + 2 * K_BYTES + 2 * VT_BYTES);

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int n = lane & 31, g = lane >> 5;
  const int row_block = gridDim.x - 1 - blockIdx.x;  // late (heavier) rows first
  const int kvh = blockIdx.y;
  const int split = blockIdx.z;

  // ---- this lane's query row ----
  const int64_t r = (int64_t)row_block * BM + wave * 32 + n;
  const bool row_ok = r < p.rows;
  const int64_t token = row_ok ? r / p.group : 0;
  const int hg = row_ok ? (int)(r - token * p.group) : 0;
  const int64_t row_lin = (token * p.n_kv_heads + kvh) * p.group + hg;  // index into [tokens, N_H]
  const int32_t qp = row_ok ? p.q_pos[token] : CP_POS_PAD_Q;

  bf16x8_t qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (row_ok) t = *(const uint4*)(p.q + row_lin * D + ks * 16 + g * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, t);
  }

  // ---- query position range of the wavefront and of the workgroup ----
  int w_qmin = row_ok ? qp : INT32_MAX, w_qmax = qp;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    w_qmin = min(w_qmin, __shfl_xor(w_qmin, o, 64));
    w_qmax = max(w_qmax, __shfl_xor(w_qmax, o, 64));
  }
  if (lane == 0) {
    wg_minmax[wave * 2] = w_qmin;
    wg_minmax[wave * 2 + 1] = w_qmax;
  }
  __syncthreads();
  int wg_qmax = INT32_MIN;
#pragma unroll
  for (int w = 0; w < NWAVE; ++w) wg_qmax = max(wg_qmax, wg_minmax[w * 2 + 1]);

  // ---- KV tile range of this split ----
  const int t_begin = split * p.tiles_per_split;
  const int t_end = min(p.n_tiles, t_begin + p.tiles_per_split);
  auto next_live = [&](int t) {
    while (t < t_end && p.bounds[t].x > wg_qmax) ++t;  // smallest key position beyond every query
    return t;
  };

  float m_run = -INFINITY;  // running max of scaled scores (log2 domain)
  float l_run = 0.f;        // running denominator over this lane's half of the keys
  floatx16_t o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;

  TileRegs regs;
  int t = next_live(t_begin);
  int buf = 0;
  if (t < t_end) {
    load_tile(p, kvh, t, tid, regs);
    store_tile(kbuf0, vtbuf0, tid, regs);
  }
  __syncthreads();

  while (t < t_end) {
    const int tn = next_live(t + 1);
    if (tn < t_end) load_tile(p, kvh, tn, tid, regs);

    const int2 bnd = p.bounds[t];
    const bool tail = (t + 1) * BN > p.total_kv;
    if (bnd.x <= w_qmax) {  // otherwise every key of the tile is beyond this wavefront's queries
      const char* kb = kbuf0 + buf * K_BYTES;
      const char* vb = vtbuf0 + buf * VT_BYTES;

      // S^T = K Q^T : two blocks of 32 keys x 32 queries
      floatx16_t s[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) s[0][i] = s[1][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8_t a0 = *(const bf16x8_t*)(kb + n * K_STRIDE + ks * 32 + g * 16);
        const bf16x8_t a1 = *(const bf16x8_t*)(kb + (32 + n) * K_STRIDE + ks * 32 + g * 16);
        s[0] = mfma32(a0, qf[ks], s[0]);
        s[1] = mfma32(a1, qf[ks], s[1]);
      }

      // causal mask, only where a key position can exceed a query position
      if (bnd.y > w_qmin || tail) {
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = t * BN + kb2 * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
            const int32_t kp = key < p.total_kv ? p.kv_pos[key] : CP_POS_PAD_KV;
            if (kp > qp) s[kb2][i] = -INFINITY;
          }
      }

      // online softmax in the log2 domain
      float mx = -INFINITY;
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb2][i]);
      mx = fmaxf(mx, xor32(mx));
      const float m_new = fmaxf(m_run, mx * p.scale_log2);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      float lsum = 0.f;
      bf16x8_t pb[4];
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(fmaf(s[kb2][i], p.scale_log2, -m_use));
          lsum += e;
          pb[kb2 * 2 + (i >> 3)][i & 7] = static_cast<bf16_t>(e);
        }
      l_run = fmaf(l_run, alpha, lsum);
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;

      // O^T += V^T P^T : 4 blocks of 32 channels, 4 steps of 16 keys
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const bf16x8_t a = *(const bf16x8_t*)(vb + (db * 32 + n) * VT_STRIDE + kk * 32 + g * 16);
          o_acc[db] = mfma32(a, pb[kk], o_acc[db]);
        }
    }

    if (tn < t_end)
      store_tile(kbuf0 + (buf ^ 1) * K_BYTES, vtbuf0 + (buf ^ 1) * VT_BYTES, tid, regs);
    __syncthreads();
    t = tn;
    buf ^= 1;
  }

  // ---- epilogue ----
  const float l_tot = l_run + xor32(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse_val =
      l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  if (!row_ok) return;
  if (p.n_splits == 1) {
    TO* o = (TO*)p.out + row_lin * D;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int d0 = 4 * ((i >> 2) * 8 + g * 4 + (i & 3));  // accumulator row m holds d = 4m + db
      if constexpr (sizeof(TO) == 4) {
        floatx4_t w = {o_acc[0][i] * inv, o_acc[1][i] * inv, o_acc[2][i] * inv, o_acc[3][i] * inv};
        *(floatx4_t*)((float*)o + d0) = w;
      } else {
        bf16x4_t w;
#pragma unroll
        for (int db = 0; db < 4; ++db) w[db] = static_cast<bf16_t>(o_acc[db][i] * inv);
        *(bf16x4_t*)((bf16_t*)o + d0) = w;
      }
    }
    if (g == 0) p.lse[row_lin] = lse_val;
  } else {
    float* o = p.part_out + ((int64_t)split * p.rows_all_heads + row_lin) * D;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int d0 = 4 * ((i >> 2) * 8 + g * 4 + (i & 3));
      floatx4_t w = {o_acc[0][i] * inv, o_acc[1][i] * inv, o_acc[2][i] * inv, o_acc[3][i] * inv};
      *(floatx4_t*)(o + d0) = w;
    }
    if (g == 0) p.part_lse[(int64_t)split * p.rows_all_heads + row_lin] = lse_val;
  }
}

struct Plan {
  int n_tiles, n_row_blocks, n_splits, tiles_per_split;
  size_t bounds_bytes, part_out_bytes, part_lse_bytes;
};

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

Plan make_plan(const cp_shape& s) {
  Plan pl;
  const int group = s.n_q_heads / s.n_kv_heads;
  const int64_t rows = s.total_q * group;
  pl.n_tiles = (int)((s.total_kv + BN - 1) / BN);
  pl.n_row_blocks = (int)((rows + BM - 1) / BM);
  // Split the KV axis when the row blocks alone cannot occupy the 256 CUs. Every split
  // costs one fp32 partial of the output, so keep at least 8 tiles (512 keys) per split.
  const int64_t wgs = (int64_t)pl.n_row_blocks * s.n_kv_heads;
  int splits = 1;
  if (wgs > 0 && wgs < 128 && pl.n_tiles >= 16) {
    splits = (int)std::min<int64_t>((256 + wgs - 1) / wgs, pl.n_tiles / 8);
    splits = std::max(1, std::min(splits, CP_MAX_PARTS));
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
  return round256((size_t)std::max<int64_t>((total_kv + BN - 1) / BN, 1) * sizeof(int2));
}

int launch_kv_tile_bounds(const int32_t* kv_pos, int64_t total_kv, void* bounds_out,
                          hipStream_t stream) {
  const int n_tiles = (int)((total_kv + BN - 1) / BN);
  if (n_tiles == 0) return CP_OK;
  hipLaunchKernelGGL(kv_tile_bounds_kernel, dim3((n_tiles + 3) / 4), dim3(256), 0, stream, kv_pos,
                     (int32_t)total_kv, n_tiles, (int2*)bounds_out);
  return check_launch();
}

int launch_prefill_mfma(const cp_shape& s, float scale, const void* q, const void* k,
                        const void* v, const int32_t* q_pos, const int32_t* kv_pos, void* out,
                        float* lse, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                        const void* tile_bounds, hipStream_t stream) {
  const Plan pl = make_plan(s);
  if (workspace_bytes < pl.bounds_bytes + pl.part_out_bytes + pl.part_lse_bytes)
    return CP_ERR_WORKSPACE;
  if (pl.n_row_blocks == 0) return CP_OK;
  if (s.n_kv_heads > 65535 || pl.n_splits > 65535) return CP_ERR_SHAPE;

  char* ws = (char*)workspace;
  Params p;
  p.q = (const bf16_t*)q; p.k = (const bf16_t*)k; p.v = (const bf16_t*)v;
  p.q_pos = q_pos; p.kv_pos = kv_pos;
  p.bounds = tile_bounds != nullptr ? (const int2*)tile_bounds : (const int2*)ws;
  p.out = out; p.lse = lse;
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
  auto kern = direct_bf16 ? prefill_mfma_kernel<bf16_t> : prefill_mfma_kernel<float>;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                          SMEM_BYTES) != hipSuccess)
    return CP_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), SMEM_BYTES, stream, p);
  if (check_launch() != CP_OK) return CP_ERR_LAUNCH;

  if (pl.n_splits > 1)
    return launch_merge_strided(p.rows_all_heads, D, pl.n_splits, p.part_out, p.part_lse,
                                p.rows_all_heads, out, out_dtype, lse, stream);
  return CP_OK;
}

}  // namespace cp
