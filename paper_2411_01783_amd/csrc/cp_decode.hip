// Split-KV decode attention for gfx950 (Algorithm 4: GQA(Q^s_k, KV_k[bid^s_k])).
//
// One query token per sequence, bf16, head_dim 128. The work is bound by reading
// K and V once from HBM: 512 bytes and 512*G flops per KV token for a group of G
// query heads, so the products run on MFMA with the G <= 16 heads as the N side
// of v_mfma_f32_16x16x32_bf16 and the keys as the M side (S^T = K Q^T, then
// O^T += V^T P^T), which keeps the softmax statistics per lane.
//
// grid = (n_splits, n_queries, n_kv_heads), sized so that all workgroups are
// resident at once (two workgroups of 4 wavefronts per CU). A workgroup takes one
// contiguous slice of the query's KV segment; its wavefronts take 32-key tiles
// round-robin, each staging its tile through a private LDS region (K swizzled, V
// transposed on the way in; every HBM read is a full 256-byte row per 16 lanes,
// the next tile is prefetched into registers while the current one is used).
// The four wavefront results are combined in LDS and written as one fp32
// partial (O, LSE) per split; Equation 4 over the splits finishes the call.
#include "cp_common.h"

namespace cp {
namespace {

constexpr int D = 128;
constexpr int TILE = 32;            // keys per wavefront tile
constexpr int NWAVE = 4;
constexpr int NTHREADS = NWAVE * 64;
constexpr int K_TILE_BYTES = TILE * D * 2;      // 8 KiB, rows of 256 B, 16-byte chunks xor-swizzled
constexpr int VT_STRIDE = TILE * 2 + 16;        // 80 B per channel row (32 keys + pad)
constexpr int VT_TILE_BYTES = D * VT_STRIDE;    // 10 KiB
constexpr int WAVE_LDS = K_TILE_BYTES + VT_TILE_BYTES;
constexpr int CB_STRIDE = D + 4;                // combine buffer: one head row of O + pad (floats)
constexpr int CB_WAVE = 16 * CB_STRIDE + 32;    // 16 heads + (m, l) per wavefront (floats)
static_assert(NWAVE * WAVE_LDS >= NWAVE * CB_WAVE * 4, "combine buffer aliases the tile buffers");

struct Params {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  const int32_t* q_pos;
  const int32_t* kv_pos;
  const int32_t* cu_kv;
  const int32_t* bid;
  float* part_out;  // [n_splits][n_q * n_q_heads][D]
  float* part_lse;  // [n_splits][n_q * n_q_heads]
  int32_t n_q;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t group;
  int32_t n_splits;
  float scale_log2;
};

__device__ __forceinline__ floatx4_t mfma16(bf16x8_t a, bf16x8_t b, floatx4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// One 32-key tile in flight: 8 x 16 B of K and 8 x 16 B of V per lane (scalars, not arrays).
struct TileRegs {
  uint4 k0, k1, k2, k3, k4, k5, k6, k7;  // row it*4 + lane/16, chunk lane%16
  uint4 v0, v1, v2, v3, v4, v5, v6, v7;  // it = 0,1: keys (lane/16 + 4*it)*4 + b, channels (lane%16)*8..+7
  int32_t p0, p1, p2, p3, p4, p5, p6, p7;  // kv_pos of keys kb*16 + (lane/16)*4 + i (this lane's scores)
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// K and V are read exactly once: streaming (non-temporal) loads
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)p));
}

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}


__global__ __launch_bounds__(NTHREADS, 2) void decode_kernel(Params p) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int hd = lane & 15;   // query head within the group (N side)
  const int kg = lane >> 4;   // key / channel sub-group
  const int split = blockIdx.x, qi = blockIdx.y, kvh = blockIdx.z;
  char* const kbuf = smem + wave * WAVE_LDS;
  char* const vtbuf = kbuf + K_TILE_BYTES;

  // segment of this query's sequence, this workgroup's slice of it
  const int b = p.bid[qi];
  const int32_t qp = p.q_pos[qi];
  // Q^T fragments (independent of the segment lookup): lane (hd, kg) holds channels
  // kg*32 + ks*8 .. +7 of head hd
  bf16x8_t qf[4];
  const bool head_ok = hd < p.group;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (head_ok)
      t = *(const uint4*)(p.q + ((int64_t)qi * p.n_q_heads + kvh * p.group + hd) * D + kg * 32 +
                          ks * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, t);
  }
  const int64_t seg0 = p.cu_kv[b], seg1 = p.cu_kv[b + 1];
  const int64_t len = seg1 - seg0;
  int64_t chunk = (len + p.n_splits - 1) / p.n_splits;
  chunk = (chunk + TILE - 1) / TILE * TILE;
  const int64_t c0 = seg0 + (int64_t)split * chunk;
  const int64_t c1 = min(seg1, c0 + chunk);

  // per-lane element offsets inside a tile (the tile base is wave-uniform)
  const uint32_t tok_stride = (uint32_t)p.n_kv_heads * D;
  const uint32_t koff = (uint32_t)(lane >> 4) * tok_stride + kvh * D + (lane & 15) * 8;
  const uint32_t voff = (uint32_t)(lane >> 4) * 4 * tok_stride + kvh * D + (lane & 15) * 8;

  float m_run = -INFINITY, l_run = 0.f;
  floatx4_t o_acc[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) o_acc[db] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  TileRegs r;
  // Rows past the end of the slice are clamped to its last row: their scores are masked
  // (position = pad) and their finite V rows meet P = 0.
  auto load_tile = [&](int64_t key0) {
    const int n_valid = (int)min<int64_t>(TILE, c1 - key0);
    const bf16_t* kt = p.k + key0 * tok_stride;
    const bf16_t* vt = p.v + key0 * tok_stride;
    {
      const int32_t* pp = p.kv_pos + key0;
      const int last = n_valid - 1, q4 = (lane >> 4) * 4;
      auto pos = [&](int kk) { return kk <= last ? pp[kk] : CP_POS_PAD_KV; };
      r.p0 = pos(q4); r.p1 = pos(q4 + 1); r.p2 = pos(q4 + 2); r.p3 = pos(q4 + 3);
      r.p4 = pos(16 + q4); r.p5 = pos(17 + q4); r.p6 = pos(18 + q4); r.p7 = pos(19 + q4);
    }
    if (n_valid == TILE) {
      r.k0 = load_stream16(kt + koff);
      r.k1 = load_stream16(kt + koff + 4 * tok_stride);
      r.k2 = load_stream16(kt + koff + 8 * tok_stride);
      r.k3 = load_stream16(kt + koff + 12 * tok_stride);
      r.k4 = load_stream16(kt + koff + 16 * tok_stride);
      r.k5 = load_stream16(kt + koff + 20 * tok_stride);
      r.k6 = load_stream16(kt + koff + 24 * tok_stride);
      r.k7 = load_stream16(kt + koff + 28 * tok_stride);
      r.v0 = load_stream16(vt + voff);
      r.v1 = load_stream16(vt + voff + tok_stride);
      r.v2 = load_stream16(vt + voff + 2 * tok_stride);
      r.v3 = load_stream16(vt + voff + 3 * tok_stride);
      r.v4 = load_stream16(vt + voff + 16 * tok_stride);
      r.v5 = load_stream16(vt + voff + 17 * tok_stride);
      r.v6 = load_stream16(vt + voff + 18 * tok_stride);
      r.v7 = load_stream16(vt + voff + 19 * tok_stride);
    } else {
      const int last = n_valid - 1;
      const uint32_t col = kvh * D + (lane & 15) * 8;
      auto krow = [&](int it) {
        return load_stream16(kt + (uint32_t)min(it * 4 + (lane >> 4), last) * tok_stride + col);
      };
      auto vrow = [&](int it, int bb) {
        return load_stream16(vt + (uint32_t)min(((lane >> 4) + 4 * it) * 4 + bb, last) * tok_stride + col);
      };
      r.k0 = krow(0); r.k1 = krow(1); r.k2 = krow(2); r.k3 = krow(3);
      r.k4 = krow(4); r.k5 = krow(5); r.k6 = krow(6); r.k7 = krow(7);
      r.v0 = vrow(0, 0); r.v1 = vrow(0, 1); r.v2 = vrow(0, 2); r.v3 = vrow(0, 3);
      r.v4 = vrow(1, 0); r.v5 = vrow(1, 1); r.v6 = vrow(1, 2); r.v7 = vrow(1, 3);
    }
  };

  // K: chunk c of row `key` goes to chunk position c ^ (key & 15) (conflict-free b128 reads
  // by 16 lanes that hold 16 different keys). V: transposed; physical row (d % 8) * 16 + d / 8
  // holds channel d; key (a*16 + kq*4 + b) of the tile sits at slot kq*8 + a*4 + b, the order
  // in which two 16-key score blocks feed the B operand of the second product.
  auto store_v = [&](int it, const uint4& a0, const uint4& a1, const uint4& a2, const uint4& a3) {
    const int kq = lane >> 4;             // key quad inside the 16-key block `it`
    const int dc = lane & 15;
    const int slot0 = kq * 8 + it * 4;
    const uint32_t w0[4] = {a0.x, a0.y, a0.z, a0.w}, w1[4] = {a1.x, a1.y, a1.z, a1.w};
    const uint32_t w2[4] = {a2.x, a2.y, a2.z, a2.w}, w3[4] = {a3.x, a3.y, a3.z, a3.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // channel pair (2j, 2j+1) of this lane's 8 channels
      const uint2 lo = make_uint2((w0[j] & 0xffffu) | (w1[j] << 16), (w2[j] & 0xffffu) | (w3[j] << 16));
      const uint2 hi = make_uint2((w0[j] >> 16) | (w1[j] & 0xffff0000u),
                                  (w2[j] >> 16) | (w3[j] & 0xffff0000u));
      *(uint2*)(vtbuf + ((2 * j) * 16 + dc) * VT_STRIDE + slot0 * 2) = lo;
      *(uint2*)(vtbuf + ((2 * j + 1) * 16 + dc) * VT_STRIDE + slot0 * 2) = hi;
    }
  };
  auto store_tile = [&]() {
    const int c = lane & 15, k4 = lane >> 4;
#define CP_STORE_K(IT, REG)                                                                  \
  *(uint4*)(kbuf + ((IT) * 4 + k4) * 256 + ((c ^ (((IT) * 4 + k4) & 15)) << 4)) = REG;
    CP_STORE_K(0, r.k0) CP_STORE_K(1, r.k1) CP_STORE_K(2, r.k2) CP_STORE_K(3, r.k3)
    CP_STORE_K(4, r.k4) CP_STORE_K(5, r.k5) CP_STORE_K(6, r.k6) CP_STORE_K(7, r.k7)
#undef CP_STORE_K
    store_v(0, r.v0, r.v1, r.v2, r.v3);
    store_v(1, r.v4, r.v5, r.v6, r.v7);
  };

  int64_t key0 = c0 + (int64_t)wave * TILE;
  if (key0 < c1) load_tile(key0);

  while (key0 < c1) {
    // positions of the 8 keys whose scores this lane holds (block kb, key kg*4 + i)
    const int32_t kp[8] = {r.p0, r.p1, r.p2, r.p3, r.p4, r.p5, r.p6, r.p7};
    wave_lds_sync();  // previous tile's LDS reads are done before it is overwritten
    store_tile();
    const int64_t key_next = key0 + NWAVE * TILE;
    if (key_next < c1) load_tile(key_next);
    wave_lds_sync();

    // S^T = K Q^T for two blocks of 16 keys
    floatx4_t s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      s[kb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
      const int key = kb * 16 + hd;  // A-operand row of this lane
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int chunk_id = kg * 4 + ks;
        const bf16x8_t a =
            *(const bf16x8_t*)(kbuf + key * 256 + ((chunk_id ^ (key & 15)) << 4));
        s[kb] = mfma16(a, qf[ks], s[kb]);
      }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (kp[kb * 4 + i] > qp) s[kb][i] = -INFINITY;
        mx = fmaxf(mx, s[kb][i]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * p.scale_log2);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    float lsum = 0.f;
    bf16x8_t pb;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float e = __builtin_amdgcn_exp2f(fmaf(s[kb][i], p.scale_log2, -m_use));
        lsum += e;
        pb[kb * 4 + i] = static_cast<bf16_t>(e);
      }
    l_run = fmaf(l_run, alpha, lsum);
    m_run = m_new;
    // O^T += V^T P^T over 8 blocks of 16 channels (block db holds channels hd*8 + db)
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const bf16x8_t a = *(const bf16x8_t*)(vtbuf + (db * 16 + hd) * VT_STRIDE + kg * 16);
#pragma unroll
      for (int i = 0; i < 4; ++i) o_acc[db][i] *= alpha;
      o_acc[db] = mfma16(a, pb, o_acc[db]);
    }
    key0 = key_next;
  }

  // ---- combine the four wavefronts (disjoint key subsets) in LDS ----
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();  // all tile buffers are dead
  float* const cbuf = (float*)smem;
  float* const my = cbuf + wave * CB_WAVE;
  // accumulator (db, i) of lane (hd, kg) is O^T row m = kg*4 + i of block db: channel m*8 + db
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int d0 = (kg * 4 + i) * 8;
    floatx4_t w0 = {o_acc[0][i], o_acc[1][i], o_acc[2][i], o_acc[3][i]};
    floatx4_t w1 = {o_acc[4][i], o_acc[5][i], o_acc[6][i], o_acc[7][i]};
    *(floatx4_t*)(my + hd * CB_STRIDE + d0) = w0;
    *(floatx4_t*)(my + hd * CB_STRIDE + d0 + 4) = w1;
  }
  if (kg == 0) {
    my[16 * CB_STRIDE + hd] = m_run;
    my[16 * CB_STRIDE + 16 + hd] = l_run;
  }
  __syncthreads();
  // thread -> (head = tid / 16, channels (tid % 16) * 8 .. +7)
  {
    const int h = tid >> 4, d0 = (tid & 15) * 8;
    float mw[NWAVE], lw[NWAVE], mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) {
      mw[w] = cbuf[w * CB_WAVE + 16 * CB_STRIDE + h];
      lw[w] = cbuf[w * CB_WAVE + 16 * CB_STRIDE + 16 + h];
      mmax = fmaxf(mmax, mw[w]);
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    if (mmax != -INFINITY) {
#pragma unroll
      for (int w = 0; w < NWAVE; ++w) {
        const float f = __builtin_amdgcn_exp2f(mw[w] - mmax);
        den = fmaf(lw[w], f, den);
        const float* src = cbuf + w * CB_WAVE + h * CB_STRIDE + d0;
        const floatx4_t x0 = *(const floatx4_t*)src, x1 = *(const floatx4_t*)(src + 4);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          acc[c] = fmaf(x0[c], f, acc[c]);
          acc[4 + c] = fmaf(x1[c], f, acc[4 + c]);
        }
      }
    }
    if (h < p.group) {
      const int64_t row = (int64_t)qi * p.n_q_heads + kvh * p.group + h;
      const int64_t prow = (int64_t)split * p.n_q * p.n_q_heads + row;
      const float inv = den > 0.f ? 1.f / den : 0.f;
      float* o = p.part_out + prow * D + d0;
      floatx4_t w0 = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
      floatx4_t w1 = {acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv};
      *(floatx4_t*)o = w0;
      *(floatx4_t*)(o + 4) = w1;
      if ((tid & 15) == 0)
        p.part_lse[prow] = den > 0.f ? (mmax + __builtin_amdgcn_logf(den)) * kLn2 : -INFINITY;
    }
  }
}

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// Power-of-two split count: about 512 workgroups in total (two per CU, all resident at
// once), at least 128 keys per split on average.
int plan_splits(const cp_shape& s) {
  const int64_t wg_per_split = std::max<int64_t>(1, s.total_q * s.n_kv_heads);
  const int64_t avg_len = s.batch > 0 ? s.total_kv / s.batch : 0;
  int splits = 1;
  while (splits < CP_MAX_PARTS && wg_per_split * splits * 2 <= 512 &&
         (int64_t)splits * 2 * 128 <= avg_len)
    splits *= 2;
  return splits;
}

}  // namespace

size_t decode_workspace_bytes(const cp_shape& s) {
  const int splits = plan_splits(s);
  const size_t rows = (size_t)s.total_q * s.n_q_heads;
  return round256(splits * rows * D * 4) + round256(splits * rows * 4);
}

int launch_decode(const cp_shape& s, float scale, const void* q, const void* k, const void* v,
                  const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_kv,
                  const int32_t* bid, void* out, float* lse, int32_t out_dtype, void* workspace,
                  size_t workspace_bytes, hipStream_t stream) {
  const int splits = plan_splits(s);
  const size_t rows = (size_t)s.total_q * s.n_q_heads;
  const size_t out_bytes = round256(splits * rows * D * 4);
  if (workspace_bytes < out_bytes + round256(splits * rows * 4)) return CP_ERR_WORKSPACE;
  if (s.total_q > 65535 || s.n_kv_heads > 65535) return CP_ERR_SHAPE;
  // per-lane offsets inside a 32-key tile are kept in 32 bits
  if ((int64_t)s.n_kv_heads * D * 64 > 0x7fffffffLL) return CP_ERR_SHAPE;

  Params p;
  p.q = (const bf16_t*)q; p.k = (const bf16_t*)k; p.v = (const bf16_t*)v;
  p.q_pos = q_pos; p.kv_pos = kv_pos; p.cu_kv = cu_kv; p.bid = bid;
  p.part_out = (float*)workspace;
  p.part_lse = (float*)((char*)workspace + out_bytes);
  p.n_q = (int32_t)s.total_q;
  p.n_q_heads = s.n_q_heads; p.n_kv_heads = s.n_kv_heads;
  p.group = s.n_q_heads / s.n_kv_heads;
  p.n_splits = splits;
  p.scale_log2 = scale * kLog2e;

  const int smem = NWAVE * WAVE_LDS;
  if (hipFuncSetAttribute((const void*)decode_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                          smem) != hipSuccess)
    return CP_ERR_LAUNCH;
  hipLaunchKernelGGL(decode_kernel, dim3(splits, (unsigned)s.total_q, s.n_kv_heads),
                     dim3(NTHREADS), smem, stream, p);
  if (check_launch() != CP_OK) return CP_ERR_LAUNCH;
  return launch_merge_strided((int64_t)rows, D, splits, p.part_out, p.part_lse, (int64_t)rows,
                              out, out_dtype, lse, stream);
}

}  // namespace cp

