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
//     and walks the KV axis in tiles of 128 keys staged through LDS (double
//     buffered; K as [key][d], V transposed to [d][key] while it is stored),
//     one workgroup barrier per tile. A tile is consumed in two steps of 64 keys.
//   - Scores are produced transposed, S^T = K Q^T with v_mfma_f32_32x32x16_bf16:
//     a lane then holds 16 keys of ONE query per 32-key block, so the softmax
//     row statistics are per-lane scalars (one cross-lane exchange with lane^32)
//     and the exponentiated block is already in the B-operand layout of the
//     second product O^T += V^T P^T. No register shuffle between the products.
//   - The next tile travels HBM/L2 -> registers -> LDS in two halves while the
//     current one is computed; the LDS stores sit between the softmax and the
//     second product, when the LDS pipe is otherwise idle.
//   - Tile skipping (load-balanced sharding leaves half of every off-diagonal
//     step fully masked): a pre-pass records min/max kv_pos of every KV tile;
//     each workgroup compacts the tiles any of its queries can see into a list
//     in LDS and walks only those; only tiles that straddle a query position
//     pay for the mask.
//   - Short query shards (pass-Q partial prefill) are split over the KV axis
//     (grid.z); split results go to the workspace and are combined with Eq. 4.
//   - The epilogue transposes the accumulators through LDS so that every output
//     row leaves as one contiguous 512-byte (fp32) or 256-byte (bf16) run.
#include "cp_common.h"

namespace cp {
namespace {

constexpr int D = 128;          // head_dim
constexpr int BM = 256;         // rows per workgroup
constexpr int TILE = 128;       // keys per LDS tile (one barrier)
constexpr int SUB = 64;         // keys per compute step
constexpr int NWAVE = 8;        // wavefronts per workgroup
constexpr int NTHREADS = NWAVE * 64;
constexpr int K_STRIDE = D * 2 + 16;      // bytes per key row in LDS (+16: conflict-free b128 reads)
constexpr int VT_STRIDE = TILE * 2 + 16;  // bytes per channel row of transposed V
constexpr int K_BYTES = TILE * K_STRIDE;
constexpr int VT_BYTES = D * VT_STRIDE;
constexpr int POS_BYTES = TILE * 4;
constexpr int MAX_LIVE = 512;   // live-tile list entries per chunk (8 wavefronts x 64 tiles)
constexpr int OFF_VT = 2 * K_BYTES;
constexpr int OFF_POS = OFF_VT + 2 * VT_BYTES;
constexpr int OFF_SCRATCH = OFF_POS + 2 * POS_BYTES;
constexpr int OFF_LIVE = OFF_SCRATCH + 128;  // scratch: 8 maxima, 1 count, 8 minima (ints)
constexpr int SMEM_BYTES = OFF_LIVE + MAX_LIVE * 16;
constexpr int OUT_STRIDE = D * 4 + 16;    // epilogue staging: one fp32 output row + pad
static_assert(NWAVE * 32 * OUT_STRIDE <= OFF_POS, "epilogue staging aliases the tile buffers");
static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget of one CU");
constexpr float kRescaleSlack = 8.f;  // log2 units
constexpr int kReadAhead = 8;
#ifndef CP_DL_READ_AHEAD_V
#define CP_DL_READ_AHEAD_V 4
#endif
constexpr int kReadAheadV = CP_DL_READ_AHEAD_V;  // V^T fragments (two transposed reads each) in flight
#ifndef CP_MIN_TILES_PER_SPLIT
#define CP_MIN_TILES_PER_SPLIT 1
#endif
constexpr int kMinTilesPerSplit = CP_MIN_TILES_PER_SPLIT;         // LDS fragment reads in flight ahead of their MFMA

struct Params {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  const int32_t* q_pos;
  const int32_t* kv_pos;
  const int32_t* q_lo;    // BAND only: smallest visible key position per query token
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

// Global -> register staging of half a KV tile (64 keys), held while the current tile is
// computed. Scalars, not arrays: keeps them out of scratch.
struct HalfRegs {
  uint4 k0, k1;          // 2 x 8 bf16 of K
  uint2 v0, v1, v2, v3;  // 4 keys x 4 bf16 of V
  int32_t pos;           // kv_pos of key `tid` of the half (first wavefront only)
};

// Per-thread element offsets of its loads inside a half tile; the base is wave-uniform.
struct HalfOffsets {
  uint32_t k[2];
  uint32_t v[4];
};

__device__ __forceinline__ HalfOffsets half_offsets(const Params& p, int kvh, int tid) {
  HalfOffsets o;
  const uint32_t tok_stride = (uint32_t)p.n_kv_heads * D;
  const uint32_t head_off = (uint32_t)kvh * D;
#pragma unroll
  for (int pp = 0; pp < 2; ++pp)
    o.k[pp] = (pp * 32 + (tid >> 4)) * tok_stride + head_off + (tid & 15) * 8;
#pragma unroll
  for (int b = 0; b < 4; ++b)
    o.v[b] = ((tid >> 5) * 4 + b) * tok_stride + head_off + (tid & 31) * 4;
  return o;
}

__device__ __forceinline__ void load_half(const Params& p, const HalfOffsets& off, int kvh,
                                          int key0, int tid, HalfRegs& r) {
  const int64_t tok_stride = (int64_t)p.n_kv_heads * D;
  if (key0 + SUB <= p.total_kv) {  // whole half inside the shard (uniform branch)
    const bf16_t* kt = p.k + key0 * tok_stride;
    const bf16_t* vt = p.v + key0 * tok_stride;
    r.k0 = *(const uint4*)(kt + off.k[0]);
    r.k1 = *(const uint4*)(kt + off.k[1]);
    r.v0 = *(const uint2*)(vt + off.v[0]);
    r.v1 = *(const uint2*)(vt + off.v[1]);
    r.v2 = *(const uint2*)(vt + off.v[2]);
    r.v3 = *(const uint2*)(vt + off.v[3]);
    if (tid < SUB) r.pos = p.kv_pos[key0 + tid];
    return;
  }
  // Tail: rows past the end of the shard are clamped to the last row. Their scores are
  // masked (the tail tile always takes the mask path, and their position is the pad
  // value) and their finite V rows meet P = 0.
  const int last = p.total_kv - 1;
  const int64_t head_off = (int64_t)kvh * D;
  auto krow = [&](int pp) {
    const int key = min(key0 + pp * 32 + (tid >> 4), last);
    return *(const uint4*)(p.k + key * tok_stride + head_off + (tid & 15) * 8);
  };
  auto vrow = [&](int b) {
    const int key = min(key0 + (tid >> 5) * 4 + b, last);
    return *(const uint2*)(p.v + key * tok_stride + head_off + (tid & 31) * 4);
  };
  r.k0 = krow(0); r.k1 = krow(1);
  r.v0 = vrow(0); r.v1 = vrow(1); r.v2 = vrow(2); r.v3 = vrow(3);
  if (tid < SUB) r.pos = key0 + tid <= last ? p.kv_pos[key0 + tid] : CP_POS_PAD_KV;
}

// Register -> LDS for half `h` of a tile buffer. K keeps its [key][d] layout. V is
// transposed: physical row rho = (d % 4) * 32 + d / 4 holds channel d, and inside every
// block of 16 keys the key (a*8 + g*4 + b) sits at slot (g*8 + a*4 + b), which is the order
// in which the accumulator of S^T hands the probabilities to the second product.
__device__ __forceinline__ void store_half(char* kbuf, char* vtbuf, int32_t* posbuf, int h,
                                           int tid, const HalfRegs& r) {
  if (tid < SUB) posbuf[h * SUB + tid] = r.pos;
  char* kh = kbuf + h * SUB * K_STRIDE;
  *(uint4*)(kh + (tid >> 4) * K_STRIDE + (tid & 15) * 16) = r.k0;
  *(uint4*)(kh + (32 + (tid >> 4)) * K_STRIDE + (tid & 15) * 16) = r.k1;
  const int kq = tid >> 5, dc = tid & 31;
  const int blk = kq >> 2, a = (kq & 3) >> 1, g = kq & 1;
  const int slot0 = h * SUB + blk * 16 + g * 8 + a * 4;
  const uint32_t x0 = r.v0.x, x1 = r.v1.x, x2 = r.v2.x, x3 = r.v3.x;
  const uint32_t y0 = r.v0.y, y1 = r.v1.y, y2 = r.v2.y, y3 = r.v3.y;
  uint2 t[4];
  t[0] = make_uint2((x0 & 0xffffu) | (x1 << 16), (x2 & 0xffffu) | (x3 << 16));
  t[1] = make_uint2((x0 >> 16) | (x1 & 0xffff0000u), (x2 >> 16) | (x3 & 0xffff0000u));
  t[2] = make_uint2((y0 & 0xffffu) | (y1 << 16), (y2 & 0xffffu) | (y3 << 16));
  t[3] = make_uint2((y0 >> 16) | (y1 & 0xffff0000u), (y2 >> 16) | (y3 & 0xffff0000u));
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *(uint2*)(vtbuf + (i * 32 + dc) * VT_STRIDE + slot0 * 2) = t[i];
}

// BAND: packed batch. Positions are shifted per sequence and a query also has a lower bound
// q_lo (the shift of its sequence): visible iff q_lo <= kv_pos <= q_pos.
template <typename TO, bool BAND>
__global__ __launch_bounds__(NTHREADS) void prefill_mfma_kernel(
    Params p, const int2* __restrict__ tile_bounds) {
  // tile_bounds is a separate read-only, non-aliased argument so that it is fetched
  // without touching the counters the tile prefetch depends on.
  extern __shared__ __align__(16) char smem[];
  char* const kbuf0 = smem;
  char* const vtbuf0 = smem + OFF_VT;
  int32_t* const posbuf0 = (int32_t*)(smem + OFF_POS);
  int* const wg_scratch = (int*)(smem + OFF_SCRATCH);
  int4* const live = (int4*)(smem + OFF_LIVE);

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
  const int32_t ql = BAND && row_ok ? p.q_lo[token] : INT32_MIN;

  bf16x8_t qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (row_ok) t = *(const uint4*)(p.q + row_lin * D + ks * 16 + g * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, t);
  }

  // ---- query position range of the wavefront and of the workgroup ----
  int w_qmin = row_ok ? qp : INT32_MAX, w_qmax = qp;
  // lower bounds of the rows that can see anything (a padded query has the empty range)
  const bool sees = row_ok && qp >= 0;
  int w_lomin = BAND && sees ? ql : INT32_MAX, w_lomax = BAND && sees ? ql : INT32_MIN;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    w_qmin = min(w_qmin, __shfl_xor(w_qmin, o, 64));
    w_qmax = max(w_qmax, __shfl_xor(w_qmax, o, 64));
    if (BAND) {
      w_lomin = min(w_lomin, __shfl_xor(w_lomin, o, 64));
      w_lomax = max(w_lomax, __shfl_xor(w_lomax, o, 64));
    }
  }
  if (lane == 0) {
    wg_scratch[wave] = w_qmax;
    if (BAND) wg_scratch[NWAVE + 1 + wave] = w_lomin;
  }
  __syncthreads();
  int wg_qmax = INT32_MIN, wg_lomin = INT32_MAX;
#pragma unroll
  for (int w = 0; w < NWAVE; ++w) {
    wg_qmax = max(wg_qmax, wg_scratch[w]);
    if (BAND) wg_lomin = min(wg_lomin, wg_scratch[NWAVE + 1 + w]);
  }
  if (BAND) {
    wg_lomin = __builtin_amdgcn_readfirstlane(wg_lomin);
    w_lomin = __builtin_amdgcn_readfirstlane(w_lomin);
    w_lomax = __builtin_amdgcn_readfirstlane(w_lomax);
  }
  // wave-uniform by construction; say so, so that control flow stays on the scalar unit
  wg_qmax = __builtin_amdgcn_readfirstlane(wg_qmax);
  w_qmin = __builtin_amdgcn_readfirstlane(w_qmin);
  w_qmax = __builtin_amdgcn_readfirstlane(w_qmax);

  float m_run = -INFINITY;  // reference max of scaled scores (log2 domain)
  float l_run = 0.f;        // running denominator over this lane's half of the keys
  floatx16_t o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;

  HalfRegs regs;
  const HalfOffsets hoff = half_offsets(p, kvh, tid);
  const int k_off = n * K_STRIDE + g * 16;   // this lane's A-operand row of K
  const int v_off = n * VT_STRIDE + g * 16;  // and of V^T

  // ---- KV tile range of this split, walked in chunks of at most MAX_LIVE tiles ----
  const int t_begin = split * p.tiles_per_split;
  const int t_end = min(p.n_tiles, t_begin + p.tiles_per_split);
  for (int c0 = t_begin; c0 < t_end; c0 += MAX_LIVE) {
    // Compact the tiles some query of the workgroup can see (smallest key position not
    // beyond the largest query position) into an ascending list in LDS: (tile, min, max).
    __syncthreads();  // previous chunk (list, tile buffers) fully consumed
    {
      const int t = c0 + wave * 64 + lane;
      int2 b = make_int2(0, 0);
      bool lv = false;
      if (t < t_end) {
        b = tile_bounds[t];
        lv = b.x <= wg_qmax && (!BAND || b.y >= wg_lomin);
      }
      const uint64_t mask = __builtin_amdgcn_ballot_w64(lv);
      if (lane == 0) wg_scratch[wave] = __builtin_popcountll(mask);
      __syncthreads();
      int base = 0, total = 0;
#pragma unroll
      for (int w = 0; w < NWAVE; ++w) {
        const int c = wg_scratch[w];
        if (w < wave) base += c;
        total += c;
      }
      if (lv)
        live[base + __builtin_popcountll(mask & ((1ull << lane) - 1ull))] =
            make_int4(t, b.x, b.y, 0);
      if (tid == 0) wg_scratch[NWAVE] = total;
    }
    __syncthreads();
    const int n_live = __builtin_amdgcn_readfirstlane(wg_scratch[NWAVE]);
    if (n_live == 0) continue;

    // prologue: first live tile into buffer 0
    {
      const int key0 = __builtin_amdgcn_readfirstlane(live[0].x) * TILE;
      load_half(p, hoff, kvh, key0, tid, regs);
      store_half(kbuf0, vtbuf0, posbuf0, 0, tid, regs);
      if (key0 + SUB < p.total_kv) {
        load_half(p, hoff, kvh, key0 + SUB, tid, regs);
        store_half(kbuf0, vtbuf0, posbuf0, 1, tid, regs);
      }
    }
    // Every global load so far (the Q fragments among them) has landed before the loop, so
    // the only loads in flight inside it are the prefetch of the next tile.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    for (int it = 0; it < n_live; ++it) {
      const int4 e = live[it];
      const int tile = __builtin_amdgcn_readfirstlane(e.x);
      const int bmin = __builtin_amdgcn_readfirstlane(e.y);
      const int bmax = __builtin_amdgcn_readfirstlane(e.z);
      const int buf = it & 1;
      const bool has_next = it + 1 < n_live;
      const int next_key0 =
          has_next ? __builtin_amdgcn_readfirstlane(live[it + 1].x) * TILE : 0;
      char* const nk = kbuf0 + (buf ^ 1) * K_BYTES;
      char* const nv = vtbuf0 + (buf ^ 1) * VT_BYTES;
      int32_t* const np = posbuf0 + (buf ^ 1) * TILE;
      // a tile whose second half starts past the end of the shard has only one half
      const bool next_two = has_next && next_key0 + SUB < p.total_kv;
      const bool two = tile * TILE + SUB < p.total_kv;
      // every key of the tile beyond this wavefront's queries: nothing to compute here
      const bool wave_live = bmin <= w_qmax && (!BAND || bmax >= w_lomin);
      const bool need_mask =
          bmax > w_qmin || (tile + 1) * TILE > p.total_kv || (BAND && bmin < w_lomax);

      if (has_next) load_half(p, hoff, kvh, next_key0, tid, regs);

#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (h == 1 && !two) break;
        floatx16_t s[2];
        bf16x8_t pb[4];
        if (wave_live) {
          const char* kb = kbuf0 + buf * K_BYTES + h * SUB * K_STRIDE + k_off;
          // S^T = K Q^T : two blocks of 32 keys x 32 queries. A fragments are requested
          // kReadAhead reads ahead of the MFMA that consumes them; the scheduling barriers
          // pin that order (the default schedule reads each fragment right before its use).
#pragma unroll
          for (int i = 0; i < 16; ++i) s[0][i] = s[1][i] = 0.f;
          bf16x8_t ka[16];
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            ka[2 * ks] = *(const bf16x8_t*)(kb + ks * 32);
            ka[2 * ks + 1] = *(const bf16x8_t*)(kb + 32 * K_STRIDE + ks * 32);
          }
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            s[0] = mfma32(ka[2 * ks], qf[ks], s[0]);
            s[1] = mfma32(ka[2 * ks + 1], qf[ks], s[1]);
          }
          __builtin_amdgcn_sched_group_barrier(0x100, kReadAhead, 0);
#pragma unroll
          for (int i = 0; i < 16 - kReadAhead; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, kReadAhead, 0);

          // causal mask, only where a key position can exceed a query position
          if (need_mask) {
            const int32_t* pb32 = posbuf0 + buf * TILE + h * SUB + g * 4;
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const int4 kp = *(const int4*)(pb32 + kb2 * 32 + q4 * 8);  // 4 consecutive keys
                if (kp.x > qp || (BAND && kp.x < ql)) s[kb2][q4 * 4 + 0] = -INFINITY;
                if (kp.y > qp || (BAND && kp.y < ql)) s[kb2][q4 * 4 + 1] = -INFINITY;
                if (kp.z > qp || (BAND && kp.z < ql)) s[kb2][q4 * 4 + 2] = -INFINITY;
                if (kp.w > qp || (BAND && kp.w < ql)) s[kb2][q4 * 4 + 3] = -INFINITY;
              }
          }

          // Online softmax in the log2 domain. The reference maximum m_run is only raised
          // (and O, l rescaled) when some row's step maximum exceeds it by more than
          // kRescaleSlack, so exponentials stay below 2^kRescaleSlack and the 64-register
          // rescale of O is skipped on almost every step; the result is unchanged because
          // numerator and denominator share the reference.
          float mx0 = fmaxf(s[0][0], s[1][0]), mx1 = fmaxf(s[0][1], s[1][1]);
#pragma unroll
          for (int i = 2; i < 16; i += 2) {
            mx0 = fmaxf(fmaxf(mx0, s[0][i]), s[1][i]);
            mx1 = fmaxf(fmaxf(mx1, s[0][i + 1]), s[1][i + 1]);
          }
          float mx = fmaxf(mx0, mx1);
          mx = fmaxf(mx, xor32(mx));
          const float m_step = mx * p.scale_log2;
          const bool raise = m_step > m_run + kRescaleSlack;  // true on the first live step
          if (__builtin_amdgcn_ballot_w64(raise) != 0) {
            const float m_new = fmaxf(m_run, m_step);
            const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));
            l_run *= alpha;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
              for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;
          }
          const float m_use = m_run == -INFINITY ? 0.f : m_run;
          // The denominator sums the unrounded exponentials: LSE must be good to 1e-3 even
          // on rows with a handful of keys, which bf16 rounding of P would not give.
          float lsum[2] = {0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            const int kb2 = kk >> 1, i0 = (kk & 1) * 8;
#pragma unroll
            for (int jj = 0; jj < 8; jj += 2) {
              const float e0 = __builtin_amdgcn_exp2f(fmaf(s[kb2][i0 + jj], p.scale_log2, -m_use));
              const float e1 =
                  __builtin_amdgcn_exp2f(fmaf(s[kb2][i0 + jj + 1], p.scale_log2, -m_use));
              lsum[(jj >> 1) & 1] += e0 + e1;
              pb[kk][jj] = static_cast<bf16_t>(e0);
              pb[kk][jj + 1] = static_cast<bf16_t>(e1);
            }
          }
          l_run += lsum[0] + lsum[1];
        }

        // The LDS pipe is idle here: park the prefetched half of the next tile in the other
        // buffer (nobody reads it before the barrier) and fetch the following half.
        if (h == 0) {
          if (has_next) {
            store_half(nk, nv, np, 0, tid, regs);
            if (next_two) load_half(p, hoff, kvh, next_key0 + SUB, tid, regs);
          }
        } else {
          if (next_two) store_half(nk, nv, np, 1, tid, regs);
        }

        if (wave_live) {
          // O^T += V^T P^T : 4 blocks of 32 channels, 4 steps of 16 keys
          const char* vb = vtbuf0 + buf * VT_BYTES + h * SUB * 2 + v_off;
          bf16x8_t va[16];
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int db = 0; db < 4; ++db)
              va[kk * 4 + db] = *(const bf16x8_t*)(vb + db * 32 * VT_STRIDE + kk * 32);
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int db = 0; db < 4; ++db) o_acc[db] = mfma32(va[kk * 4 + db], pb[kk], o_acc[db]);
          __builtin_amdgcn_sched_group_barrier(0x100, kReadAhead, 0);
#pragma unroll
          for (int i = 0; i < 16 - kReadAhead; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, kReadAhead, 0);
        }
      }
      // single-half current tile: the second half of the next tile is still in registers
      if (!two && next_two) store_half(nk, nv, np, 1, tid, regs);
      __syncthreads();
    }
  }

  // ---- epilogue ----
  const float l_tot = l_run + xor32(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse_val =
      l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  const bool direct = p.n_splits == 1;
  float* const lse_dst = direct ? p.lse : p.part_lse + (int64_t)split * p.rows_all_heads;
  if (row_ok && g == 0) lse_dst[row_lin] = lse_val;

  // Transpose through LDS (tile buffers are dead after the last barrier; each wavefront
  // uses a private region): accumulator (db, i) of lane (n, g) is channel
  // d = 4 * ((i / 4) * 8 + g * 4 + i % 4) + db of row n.
  char* const stage = smem + wave * 32 * OUT_STRIDE;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int d0 = 4 * ((i >> 2) * 8 + g * 4 + (i & 3));
    floatx4_t w = {o_acc[0][i] * inv, o_acc[1][i] * inv, o_acc[2][i] * inv, o_acc[3][i] * inv};
    *(floatx4_t*)(stage + n * OUT_STRIDE + d0 * 4) = w;
  }
  wave_lds_fence();
  const int64_t r0 = (int64_t)row_block * BM + wave * 32;
  if (direct && sizeof(TO) == 2) {
    // 4 rows per pass: 16 lanes x 8 channels each
    bf16_t* const o = (bf16_t*)p.out;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int rr = pass * 4 + (lane >> 4), c = (lane & 15) * 8;
      const int64_t rl = __shfl(row_lin, rr, 64);
      const floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      const floatx4_t b = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4 + 16);
      bf16x8_t w;
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        w[x] = static_cast<bf16_t>(a[x]);
        w[4 + x] = static_cast<bf16_t>(b[x]);
      }
      if (r0 + rr < p.rows) *(bf16x8_t*)(o + rl * D + c) = w;
    }
  } else {
    // 2 rows per pass: 32 lanes x 4 channels each
    float* const o =
        direct ? (float*)p.out : p.part_out + (int64_t)split * p.rows_all_heads * D;
#pragma unroll
    for (int pass = 0; pass < 16; ++pass) {
      const int rr = pass * 2 + (lane >> 5), c = (lane & 31) * 4;
      const int64_t rl = __shfl(row_lin, rr, 64);
      const floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      if (r0 + rr < p.rows) *(floatx4_t*)(o + rl * D + c) = a;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Direct-to-LDS variant. K and V tiles travel HBM/L2 -> LDS with global_load_lds (16 bytes
// per lane, no register staging, no LDS store instructions, no register transposes):
//   - both tiles are stored row-major [key][256 B], unpadded (a wavefront instruction
//     writes 64 x 16 B contiguously, i.e. four whole rows); bank conflicts are avoided by
//     permuting the 16-byte chunks of a row on the GLOBAL side: chunk c of K row r lands at
//     chunk position c ^ (r & 15), chunk c of V row r at c ^ ((r & 3) * 4);
//   - K fragments (rows = keys) are read with ds_read_b128 as before;
//   - V^T fragments (rows = channels, k = keys) are read with ds_read_b64_tr_b16, which
//     hands lane i of a 16-lane group element (i % 4) of what lanes 4j + i / 4 (j = 0..3)
//     of the group addressed: four lanes address four consecutive keys of a 16-channel
//     strip, and every lane receives one channel of those four keys.
// Accumulator (db, i) of lane (n, g) is channel db*32 + (i/4)*8 + g*4 + i%4 of query n.
// ---------------------------------------------------------------------------------------
#define CP_LDS_AS __attribute__((address_space(3)))
#define CP_GLB_AS __attribute__((address_space(1)))
typedef short shortx4_t __attribute__((ext_vector_type(4)));

constexpr int ROW_BYTES = D * 2;              // one K or V row in LDS
constexpr int KD_BYTES = TILE * ROW_BYTES;    // 32 KiB per tile buffer
constexpr int OFF_V8 = 2 * KD_BYTES;
constexpr int OFF_POS8 = OFF_V8 + 2 * KD_BYTES;
constexpr int OFF_SCRATCH8 = OFF_POS8 + 2 * POS_BYTES;
constexpr int OFF_LIVE8 = OFF_SCRATCH8 + 128;
constexpr int SMEM_BYTES8 = OFF_LIVE8 + MAX_LIVE * 16;
static_assert(NWAVE * 32 * OUT_STRIDE <= SMEM_BYTES8, "epilogue staging fits in the allocation");
static_assert(SMEM_BYTES8 <= 160 * 1024, "LDS budget of one CU");

__device__ __forceinline__ void load_lds16(const void* src, char* lds_dst_wave_uniform) {
  __builtin_amdgcn_global_load_lds((const CP_GLB_AS void*)src, (CP_LDS_AS void*)lds_dst_wave_uniform,
                                   16, 0, 0);
}

__device__ __forceinline__ bf16x8_t read_vt_frag(const char* a0, const char* a1) {
  const shortx4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CP_LDS_AS shortx4_t*)a0);
  const shortx4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CP_LDS_AS shortx4_t*)a1);
  typedef short shortx8_t __attribute__((ext_vector_type(8)));
  const shortx8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8_t, v);
}

template <typename TO, bool BAND>
__global__ __launch_bounds__(NTHREADS) void prefill_mfma_dl_kernel(
    Params p, const int2* __restrict__ tile_bounds) {
  extern __shared__ __align__(16) char smem[];
  char* const kbuf0 = smem;
  char* const vbuf0 = smem + OFF_V8;
  int32_t* const posbuf0 = (int32_t*)(smem + OFF_POS8);
  int* const wg_scratch = (int*)(smem + OFF_SCRATCH8);
  int4* const live = (int4*)(smem + OFF_LIVE8);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int n = lane & 31, g = lane >> 5;
  const int row_block = gridDim.x - 1 - blockIdx.x;  // late (heavier) rows first
  const int kvh = blockIdx.y;
  const int split = blockIdx.z;

  // ---- this lane's query row ----
  const int64_t r = (int64_t)row_block * BM + wave * 32 + n;
  const bool row_ok = r < p.rows;
  const int64_t token = row_ok ? r / p.group : 0;
  const int hg = row_ok ? (int)(r - token * p.group) : 0;
  const int64_t row_lin = (token * p.n_kv_heads + kvh) * p.group + hg;
  const int32_t qp = row_ok ? p.q_pos[token] : CP_POS_PAD_Q;
  const int32_t ql = BAND && row_ok ? p.q_lo[token] : INT32_MIN;

  bf16x8_t qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (row_ok) t = *(const uint4*)(p.q + row_lin * D + ks * 16 + g * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, t);
  }

  // ---- query position range of the wavefront and of the workgroup ----
  int w_qmin = row_ok ? qp : INT32_MAX, w_qmax = qp;
  const bool sees = row_ok && qp >= 0;
  int w_lomin = BAND && sees ? ql : INT32_MAX, w_lomax = BAND && sees ? ql : INT32_MIN;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    w_qmin = min(w_qmin, __shfl_xor(w_qmin, o, 64));
    w_qmax = max(w_qmax, __shfl_xor(w_qmax, o, 64));
    if (BAND) {
      w_lomin = min(w_lomin, __shfl_xor(w_lomin, o, 64));
      w_lomax = max(w_lomax, __shfl_xor(w_lomax, o, 64));
    }
  }
  if (lane == 0) {
    wg_scratch[wave] = w_qmax;
    if (BAND) wg_scratch[NWAVE + 1 + wave] = w_lomin;
  }
  __syncthreads();
  int wg_qmax = INT32_MIN, wg_lomin = INT32_MAX;
#pragma unroll
  for (int w = 0; w < NWAVE; ++w) {
    wg_qmax = max(wg_qmax, wg_scratch[w]);
    if (BAND) wg_lomin = min(wg_lomin, wg_scratch[NWAVE + 1 + w]);
  }
  wg_qmax = __builtin_amdgcn_readfirstlane(wg_qmax);
  w_qmin = __builtin_amdgcn_readfirstlane(w_qmin);
  w_qmax = __builtin_amdgcn_readfirstlane(w_qmax);
  if (BAND) {
    wg_lomin = __builtin_amdgcn_readfirstlane(wg_lomin);
    w_lomin = __builtin_amdgcn_readfirstlane(w_lomin);
    w_lomax = __builtin_amdgcn_readfirstlane(w_lomax);
  }

  float m_run = -INFINITY;  // reference max of scaled scores (log2 domain)
  float l_run = 0.f;        // running denominator over this lane's half of the keys
  floatx16_t o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;

  // ---- tile loader: this wavefront brings rows wave*16 .. wave*16+15 of K and of V, four
  // rows (1 KiB) per instruction; lane l covers row l/16 of the four, chunk position l%16 ----
  const int64_t tok_stride = (int64_t)p.n_kv_heads * D;  // elements
  const int l_row = lane >> 4, l_pos = lane & 15;
  auto issue_tile = [&](int key0, int b) {
    const int last = p.total_kv - 1;
    const bool full = key0 + TILE <= p.total_kv;  // uniform
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row_in_tile = wave * 16 + i * 4 + l_row;
      const int rsel = (i * 4 + l_row) & 15;  // row_in_tile & 15
      // rows past the end of the shard are clamped to its last row (masked by their position)
      const int64_t grow = full ? key0 + row_in_tile : min(key0 + row_in_tile, last);
      const bf16_t* krow = p.k + grow * tok_stride + kvh * D;
      const bf16_t* vrow = p.v + grow * tok_stride + kvh * D;
      char* const kd = kbuf0 + b * KD_BYTES + (wave * 16 + i * 4) * ROW_BYTES;
      char* const vd = vbuf0 + b * KD_BYTES + (wave * 16 + i * 4) * ROW_BYTES;
      load_lds16(krow + (l_pos ^ rsel) * 8, kd);
      load_lds16(vrow + (l_pos ^ ((l_row & 3) * 4)) * 8, vd);
    }
  };
  // kv_pos of the tile goes through a register (the tail needs the pad value)
  auto load_pos = [&](int key0) -> int32_t {
    if (tid >= TILE) return 0;
    const int key = key0 + tid;
    return key < p.total_kv ? p.kv_pos[key] : CP_POS_PAD_KV;
  };

  // ---- fragment addressing ----
  // K: lane (n, g) reads chunk 2*ks + g of rows n and n + 32 of a 64-key half
  int k_chunk_off[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_chunk_off[ks] = ((2 * ks + g) ^ (n & 15)) * 16;
  const int k_lane = n * ROW_BYTES;
  // V: in its 16-lane group this lane addresses key j of four and 8 bytes (4 channels) q
  const int grp = lane >> 4, vj = (lane & 15) >> 2, vq = lane & 3;
  const int v_lane = ((grp >> 1) * 4 + vj) * ROW_BYTES + (grp & 1) * 32 + (vq >> 1) * 16 + (vq & 1) * 8;
  int v_db_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) v_db_off[db] = (db ^ vj) * 64;

  const int t_begin = split * p.tiles_per_split;
  const int t_end = min(p.n_tiles, t_begin + p.tiles_per_split);
  for (int c0 = t_begin; c0 < t_end; c0 += MAX_LIVE) {
    __syncthreads();  // previous chunk (list, tile buffers) fully consumed
    {
      const int t = c0 + wave * 64 + lane;
      int2 b = make_int2(0, 0);
      bool lv = false;
      if (t < t_end) {
        b = tile_bounds[t];
        lv = b.x <= wg_qmax && (!BAND || b.y >= wg_lomin);
      }
      const uint64_t mask = __builtin_amdgcn_ballot_w64(lv);
      if (lane == 0) wg_scratch[wave] = __builtin_popcountll(mask);
      __syncthreads();
      int base = 0, total = 0;
#pragma unroll
      for (int w = 0; w < NWAVE; ++w) {
        const int c = wg_scratch[w];
        if (w < wave) base += c;
        total += c;
      }
      if (lv)
        live[base + __builtin_popcountll(mask & ((1ull << lane) - 1ull))] =
            make_int4(t, b.x, b.y, 0);
      if (tid == 0) wg_scratch[NWAVE] = total;
    }
    __syncthreads();
    const int n_live = __builtin_amdgcn_readfirstlane(wg_scratch[NWAVE]);
    if (n_live == 0) continue;

    // prologue: first live tile into buffer 0
    {
      const int key0 = __builtin_amdgcn_readfirstlane(live[0].x) * TILE;
      issue_tile(key0, 0);
      const int32_t pos = load_pos(key0);
      if (tid < TILE) posbuf0[tid] = pos;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): tile (and Q fragments) have landed
    __syncthreads();

    for (int it = 0; it < n_live; ++it) {
      const int4 e = live[it];
      const int tile = __builtin_amdgcn_readfirstlane(e.x);
      const int bmin = __builtin_amdgcn_readfirstlane(e.y);
      const int bmax = __builtin_amdgcn_readfirstlane(e.z);
      const int buf = it & 1;
      const bool has_next = it + 1 < n_live;
      const bool two = tile * TILE + SUB < p.total_kv;
      const bool wave_live = bmin <= w_qmax && (!BAND || bmax >= w_lomin);
      const bool need_mask =
          bmax > w_qmin || (tile + 1) * TILE > p.total_kv || (BAND && bmin < w_lomax);

      // the next tile flies into the other buffer while this one is computed (every
      // wavefront left that buffer behind at the barrier that ended the previous tile)
      int32_t next_pos = 0;
      if (has_next) {
        const int next_key0 = __builtin_amdgcn_readfirstlane(live[it + 1].x) * TILE;
        issue_tile(next_key0, buf ^ 1);
        next_pos = load_pos(next_key0);
      }

#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (h == 1 && !two) break;
        if (!wave_live) continue;
        floatx16_t s[2];
        bf16x8_t pb[4];
        const char* kb = kbuf0 + buf * KD_BYTES + h * SUB * ROW_BYTES + k_lane;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[0][i] = s[1][i] = 0.f;
        bf16x8_t ka[16];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          ka[2 * ks] = *(const bf16x8_t*)(kb + k_chunk_off[ks]);
          ka[2 * ks + 1] = *(const bf16x8_t*)(kb + k_chunk_off[ks] + 32 * ROW_BYTES);
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          s[0] = mfma32(ka[2 * ks], qf[ks], s[0]);
          s[1] = mfma32(ka[2 * ks + 1], qf[ks], s[1]);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, kReadAhead, 0);
#pragma unroll
        for (int i = 0; i < 16 - kReadAhead; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kReadAhead, 0);

        if (need_mask) {
          const int32_t* pb32 = posbuf0 + buf * TILE + h * SUB + g * 4;
#pragma unroll
          for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const int4 kp = *(const int4*)(pb32 + kb2 * 32 + q4 * 8);  // 4 consecutive keys
              if (kp.x > qp || (BAND && kp.x < ql)) s[kb2][q4 * 4 + 0] = -INFINITY;
              if (kp.y > qp || (BAND && kp.y < ql)) s[kb2][q4 * 4 + 1] = -INFINITY;
              if (kp.z > qp || (BAND && kp.z < ql)) s[kb2][q4 * 4 + 2] = -INFINITY;
              if (kp.w > qp || (BAND && kp.w < ql)) s[kb2][q4 * 4 + 3] = -INFINITY;
            }
        }

        // online softmax in the log2 domain with a lazily raised reference maximum
        float mx0 = fmaxf(s[0][0], s[1][0]), mx1 = fmaxf(s[0][1], s[1][1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) {
          mx0 = fmaxf(fmaxf(mx0, s[0][i]), s[1][i]);
          mx1 = fmaxf(fmaxf(mx1, s[0][i + 1]), s[1][i + 1]);
        }
        float mx = fmaxf(mx0, mx1);
        mx = fmaxf(mx, xor32(mx));
        const float m_step = mx * p.scale_log2;
        const bool raise = m_step > m_run + kRescaleSlack;  // true on the first live step
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
          const float m_new = fmaxf(m_run, m_step);
          const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));
          l_run *= alpha;
          m_run = m_new;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;
        }
        const float m_use = m_run == -INFINITY ? 0.f : m_run;
        float lsum[2] = {0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int kb2 = kk >> 1, i0 = (kk & 1) * 8;
#pragma unroll
          for (int jj = 0; jj < 8; jj += 2) {
            const float e0 = __builtin_amdgcn_exp2f(fmaf(s[kb2][i0 + jj], p.scale_log2, -m_use));
            const float e1 =
                __builtin_amdgcn_exp2f(fmaf(s[kb2][i0 + jj + 1], p.scale_log2, -m_use));
            lsum[(jj >> 1) & 1] += e0 + e1;
            pb[kk][jj] = static_cast<bf16_t>(e0);
            pb[kk][jj + 1] = static_cast<bf16_t>(e1);
          }
        }
        l_run += lsum[0] + lsum[1];

        // O^T += V^T P^T : 4 blocks of 32 channels, 4 steps of 16 keys. Slot jj of a lane's
        // k-slice is key kk*16 + (jj/4)*8 + g*4 + jj%4, the order in which S^T hands over P.
        const char* vb = vbuf0 + buf * KD_BYTES + h * SUB * ROW_BYTES + v_lane;
        bf16x8_t va[16];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            const char* a0 = vb + v_db_off[db] + kk * 16 * ROW_BYTES;
            va[kk * 4 + db] = read_vt_frag(a0, a0 + 8 * ROW_BYTES);
          }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int db = 0; db < 4; ++db) o_acc[db] = mfma32(va[kk * 4 + db], pb[kk], o_acc[db]);
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * kReadAheadV, 0);
#pragma unroll
        for (int i = 0; i < 16 - kReadAheadV; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kReadAheadV, 0);
      }
      if (has_next && tid < TILE) posbuf0[(buf ^ 1) * TILE + tid] = next_pos;
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's part of the next tile
      __syncthreads();
    }
  }

  // ---- epilogue ----
  const float l_tot = l_run + xor32(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse_val =
      l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  const bool direct = p.n_splits == 1;
  float* const lse_dst = direct ? p.lse : p.part_lse + (int64_t)split * p.rows_all_heads;
  if (row_ok && g == 0) lse_dst[row_lin] = lse_val;

  // Transpose through LDS (tile buffers are dead after the last barrier; each wavefront
  // uses a private region).
  char* const stage = smem + wave * 32 * OUT_STRIDE;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int d0 = db * 32 + i4 * 8 + g * 4;
      floatx4_t w = {o_acc[db][i4 * 4 + 0] * inv, o_acc[db][i4 * 4 + 1] * inv,
                     o_acc[db][i4 * 4 + 2] * inv, o_acc[db][i4 * 4 + 3] * inv};
      *(floatx4_t*)(stage + n * OUT_STRIDE + d0 * 4) = w;
    }
  wave_lds_fence();
  const int64_t r0 = (int64_t)row_block * BM + wave * 32;
  if (direct && sizeof(TO) == 2) {
    bf16_t* const o = (bf16_t*)p.out;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int rr = pass * 4 + (lane >> 4), c = (lane & 15) * 8;
      const int64_t rl = __shfl(row_lin, rr, 64);
      const floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      const floatx4_t b = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4 + 16);
      bf16x8_t w;
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        w[x] = static_cast<bf16_t>(a[x]);
        w[4 + x] = static_cast<bf16_t>(b[x]);
      }
      if (r0 + rr < p.rows) *(bf16x8_t*)(o + rl * D + c) = w;
    }
  } else {
    float* const o =
        direct ? (float*)p.out : p.part_out + (int64_t)split * p.rows_all_heads * D;
#pragma unroll
    for (int pass = 0; pass < 16; ++pass) {
      const int rr = pass * 2 + (lane >> 5), c = (lane & 31) * 4;
      const int64_t rl = __shfl(row_lin, rr, 64);
      const floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      if (r0 + rr < p.rows) *(floatx4_t*)(o + rl * D + c) = a;
    }
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
  pl.n_tiles = (int)((s.total_kv + TILE - 1) / TILE);
  pl.n_row_blocks = (int)((rows + BM - 1) / BM);
  // Split the KV axis when the row blocks alone cannot occupy the 256 CUs. Every split
  // costs one fp32 partial of the output, so keep at least kMinTilesPerSplit tiles per split.
  const int64_t wgs = (int64_t)pl.n_row_blocks * s.n_kv_heads;
  int splits = 1;
  if (wgs > 0 && wgs < 128 && pl.n_tiles >= 2 * kMinTilesPerSplit) {
    splits = (int)std::min<int64_t>((256 + wgs - 1) / wgs, pl.n_tiles / kMinTilesPerSplit);
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

int launch_prefill_mfma(const cp_shape& s, float scale, const void* q, const void* k,
                        const void* v, const int32_t* q_pos, const int32_t* kv_pos, void* out,
                        float* lse, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                        const void* tile_bounds, const int32_t* q_lo, hipStream_t stream) {
  const Plan pl = make_plan(s);
  if (workspace_bytes < pl.bounds_bytes + pl.part_out_bytes + pl.part_lse_bytes)
    return CP_ERR_WORKSPACE;
  if (pl.n_row_blocks == 0) return CP_OK;
  if (s.n_kv_heads > 65535 || pl.n_splits > 65535) return CP_ERR_SHAPE;

  char* ws = (char*)workspace;
  Params p;
  p.q = (const bf16_t*)q; p.k = (const bf16_t*)k; p.v = (const bf16_t*)v;
  p.q_pos = q_pos; p.kv_pos = kv_pos; p.q_lo = q_lo;
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
#ifdef CP_PREFILL_STAGED
  auto kern = q_lo != nullptr
                  ? (direct_bf16 ? prefill_mfma_kernel<bf16_t, true> : prefill_mfma_kernel<float, true>)
                  : (direct_bf16 ? prefill_mfma_kernel<bf16_t, false>
                                 : prefill_mfma_kernel<float, false>);
  constexpr int kSmem = SMEM_BYTES;
#else
  auto kern = q_lo != nullptr ? (direct_bf16 ? prefill_mfma_dl_kernel<bf16_t, true>
                                             : prefill_mfma_dl_kernel<float, true>)
                              : (direct_bf16 ? prefill_mfma_dl_kernel<bf16_t, false>
                                             : prefill_mfma_dl_kernel<float, false>);
  constexpr int kSmem = SMEM_BYTES8;
#endif
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

}  // namespace cp
