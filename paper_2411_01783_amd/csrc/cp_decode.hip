// Split-KV decode attention for gfx950 (Algorithm 4: GQA(Q^s_k, KV_k[bid^s_k])).
//
// One query token per sequence, bf16, head_dim 128. The work is bound by reading
// K and V once from HBM: 512 bytes and 512*G flops per KV token for a group of G
// query heads, so the products run on MFMA with the G <= 16 heads as the N side
// of v_mfma_f32_16x16x32_bf16 and the keys as the M side (S^T = K Q^T, then
// O^T += V^T P^T), which keeps the softmax statistics per lane.
//
// grid = (n_splits, n_queries, n_kv_heads). A workgroup of 4 wavefronts takes
// one contiguous slice of the query's KV segment; its wavefronts take 32-key
// tiles round-robin, each staging its tile through a private LDS region
// (K swizzled, V transposed on the way in; coalesced 256-byte row reads from
// HBM, the next tile prefetched into registers while the current one is used).
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
constexpr int COMBINE_BYTES = NWAVE * (16 * D + 32) * 4;  // O^T + (m, l) per wavefront
static_assert(NWAVE * WAVE_LDS >= COMBINE_BYTES, "combine buffer aliases the tile buffers");

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

struct TileRegs {
  uint4 k[8];      // 8 x 16 B of K: row it*4 + lane/16, chunk lane%16
  uint2 v[4][4];   // item it: key quad (lane/32 + 2*it), channels (lane%32)*4..+3, 4 keys
};

__device__ __forceinline__ void load_tile(const Params& p, int kvh, int64_t key0, int n_valid,
                                          int lane, TileRegs& r) {
  const int64_t tok_stride = (int64_t)p.n_kv_heads * D;
  const bf16_t* kbase = p.k + key0 * tok_stride + (int64_t)kvh * D;
  const bf16_t* vbase = p.v + key0 * tok_stride + (int64_t)kvh * D;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int key = it * 4 + (lane >> 4);
    r.k[it] = make_uint4(0, 0, 0, 0);
    if (key < n_valid) r.k[it] = *(const uint4*)(kbase + key * tok_stride + (lane & 15) * 8);
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int kq = (lane >> 5) + 2 * it;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int key = kq * 4 + b;
      r.v[it][b] = make_uint2(0, 0);
      if (key < n_valid) r.v[it][b] = *(const uint2*)(vbase + key * tok_stride + (lane & 31) * 4);
    }
  }
}

// K: chunk c of row `key` goes to chunk position c ^ (key & 15) (conflict-free b128 reads by
// 16 lanes that hold 16 different keys). V: transposed; physical row (d % 4) * 32 + d / 4
// holds channel d; key (a*16 + kg*4 + b) of the tile sits at slot kg*8 + a*4 + b, the order
// in which two 16-key score blocks feed the B operand of the second product.
__device__ __forceinline__ void store_tile(char* kbuf, char* vtbuf, int lane, const TileRegs& r) {
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int key = it * 4 + (lane >> 4);
    *(uint4*)(kbuf + key * 256 + (((lane & 15) ^ (key & 15)) << 4)) = r.k[it];
  }
  const int dc = lane & 31;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int kq = (lane >> 5) + 2 * it;           // keys kq*4 .. kq*4+3
    const int slot0 = (kq & 3) * 8 + (kq >> 2) * 4;
    const uint32_t x0 = r.v[it][0].x, x1 = r.v[it][1].x, x2 = r.v[it][2].x, x3 = r.v[it][3].x;
    const uint32_t y0 = r.v[it][0].y, y1 = r.v[it][1].y, y2 = r.v[it][2].y, y3 = r.v[it][3].y;
    uint2 t[4];
    t[0] = make_uint2((x0 & 0xffffu) | (x1 << 16), (x2 & 0xffffu) | (x3 << 16));
    t[1] = make_uint2((x0 >> 16) | (x1 & 0xffff0000u), (x2 >> 16) | (x3 & 0xffff0000u));
    t[2] = make_uint2((y0 & 0xffffu) | (y1 << 16), (y2 & 0xffffu) | (y3 << 16));
    t[3] = make_uint2((y0 >> 16) | (y1 & 0xffff0000u), (y2 >> 16) | (y3 & 0xffff0000u));
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *(uint2*)(vtbuf + (i * 32 + dc) * VT_STRIDE + slot0 * 2) = t[i];
  }
}

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(NTHREADS) void decode_kernel(Params p) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int hd = lane & 15;   // query head within the group (N side)
  const int kg = lane >> 4;   // key / channel sub-group
  const int split = blockIdx.x, qi = blockIdx.y, kvh = blockIdx.z;
  char* const kbuf = smem + wave * WAVE_LDS;
  char* const vtbuf = kbuf + K_TILE_BYTES;

  const int b = p.bid[qi];
  const int64_t seg0 = p.cu_kv[b], seg1 = p.cu_kv[b + 1];
  const int64_t len = seg1 - seg0;
  int64_t chunk = (len + p.n_splits - 1) / p.n_splits;
  chunk = (chunk + TILE - 1) / TILE * TILE;
  const int64_t c0 = seg0 + (int64_t)split * chunk;
  const int64_t c1 = min(seg1, c0 + chunk);
  const int32_t qp = p.q_pos[qi];

  // Q^T fragments: lane (hd, kg) holds channels kg*32 + ks*8 .. +7 of head hd
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

  float m_run = -INFINITY, l_run = 0.f;
  floatx4_t o_acc[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) o_acc[db] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  TileRegs regs;
  int64_t key0 = c0 + (int64_t)wave * TILE;
  if (key0 < c1) load_tile(p, kvh, key0, (int)min<int64_t>(TILE, c1 - key0), lane, regs);

  while (key0 < c1) {
    const int n_valid = (int)min<int64_t>(TILE, c1 - key0);
    wave_lds_sync();  // previous tile's LDS reads are done before it is overwritten
    store_tile(kbuf, vtbuf, lane, regs);
    const int64_t key_next = key0 + NWAVE * TILE;
    if (key_next < c1)
      load_tile(p, kvh, key_next, (int)min<int64_t>(TILE, c1 - key_next), lane, regs);
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
    // mask: lane (hd, kg) register i of block kb is key kb*16 + kg*4 + i
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kk = kb * 16 + kg * 4 + i;
        const int32_t kp = kk < n_valid ? p.kv_pos[key0 + kk] : CP_POS_PAD_KV;
        if (kp > qp) s[kb][i] = -INFINITY;
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
    // O^T += V^T P^T over 8 blocks of 16 channels
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
  float* const my = cbuf + wave * (16 * D + 32);
  // O^T accumulator (db, i) of lane (hd, kg) is physical V row rho = db*16 + kg*4 + i,
  // i.e. channel d = 4 * (rho % 32) + rho / 32
#pragma unroll
  for (int db = 0; db < 8; ++db)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rho = db * 16 + kg * 4 + i;
      const int d = 4 * (rho & 31) + (rho >> 5);
      my[hd * D + d] = o_acc[db][i];
    }
  if (kg == 0) {
    my[16 * D + hd] = m_run;
    my[16 * D + 16 + hd] = l_run;
  }
  __syncthreads();
  // thread -> (head = tid / 16, channels (tid % 16) * 8 .. +7)
  {
    const int h = tid >> 4, d0 = (tid & 15) * 8;
    float mw[NWAVE], lw[NWAVE], mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) {
      mw[w] = cbuf[w * (16 * D + 32) + 16 * D + h];
      lw[w] = cbuf[w * (16 * D + 32) + 16 * D + 16 + h];
      mmax = fmaxf(mmax, mw[w]);
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    if (mmax != -INFINITY) {
#pragma unroll
      for (int w = 0; w < NWAVE; ++w) {
        const float f = __builtin_amdgcn_exp2f(mw[w] - mmax);
        den = fmaf(lw[w], f, den);
        const float* src = cbuf + w * (16 * D + 32) + h * D + d0;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = fmaf(src[c], f, acc[c]);
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

int plan_splits(const cp_shape& s) {
  const int64_t wg_per_split = std::max<int64_t>(1, s.total_q * s.n_kv_heads);
  const int64_t avg_len = s.batch > 0 ? s.total_kv / s.batch : 0;
  int64_t splits = (768 + wg_per_split - 1) / wg_per_split;
  splits = std::min<int64_t>(splits, (avg_len + 127) / 128);
  return (int)std::max<int64_t>(1, std::min<int64_t>(splits, CP_MAX_PARTS));
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
