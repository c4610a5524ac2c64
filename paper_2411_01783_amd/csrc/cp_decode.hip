// Split-KV decode attention for gfx950 (Algorithm 4: GQA(Q^s_k, KV_k[bid^s_k])).
//
// One query token per sequence, bf16, head_dim 128. The work is bound by reading
// K and V once from HBM: 512 bytes and 512*G flops per KV token for a group of G
// query heads, so the products run on MFMA with the G <= 16 heads as the N side
// and the keys as the M side (S^T = K Q^T, then O^T += V^T P^T), which keeps the
// softmax statistics per lane.
//
// Two kernels:
//   decode_kernel       any bid. grid = (n_splits, n_queries, n_kv_heads), sized so that all
//     workgroups are resident at once (two workgroups of 4 wavefronts per CU). A workgroup
//     takes one contiguous slice of the query's KV segment; its wavefronts take 32-key tiles
//     round-robin, each staging its tile through a private LDS region (K swizzled, V
//     transposed on the way in; every HBM read is a full 256-byte row per 16 lanes, the next
//     tile is prefetched into registers while the current one is used). The four wavefront
//     results are combined in LDS and written as one fp32 partial (O, LSE) per split;
//     Equation 4 over the splits finishes the call (merge_split_kernel).
//   decode_flat_kernel  every sequence named at most once (CP_SHAPE_UNIQUE_BID): equal key
//     ranges per workgroup regardless of the sequences, direct-to-LDS loads; see below.
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

// ---------------------------------------------------------------------------
// Flat split-KV decode: the fast path for calls whose queries name every sequence at most once
// (Algorithm 4 has exactly one new token per sequence).
//
// The packed KV of the rank, [0, total_kv), is cut into equal key ranges, one per workgroup,
// regardless of where the sequences begin: a workgroup's first K/V requests then depend on
// nothing but its index, so they leave at once, and the lookups that tell it whose keys it is
// reading (cu_seqlens_kv, bid, the query, its position) complete in the shadow of that first
// round trip. The FW wavefronts of a workgroup take the range's 16-key units round-robin (a
// fixed deal: dealing them out from a counter as buffers fall free was no faster and made the
// summation order, and so the last bits of the result, vary from run to run). A
// unit goes HBM -> LDS directly (global_load_lds, no register staging), row-major with the
// 16-byte chunks of a row permuted on the global side so that the fragment reads are free of
// bank conflicts (K fragments: ds_read_b128, V^T fragments: ds_read_b64_tr_b16). Every
// wavefront keeps two units in flight, in two LDS buffers: the next one travels while the
// current one is used, and what is left after the last byte has landed is one 16-key unit.
//
// A range may hold the end of a sequence. Every wavefront then writes what it has accumulated
// for the ending sequence as a partial of its own (a "tail": slot n_main + seq * FW + wave,
// with LSE = -inf and no data if it saw nothing) and starts afresh; what the wavefronts hold
// when the range ends belongs to one sequence, is combined in LDS and becomes the workgroup's
// main partial (slot = workgroup index). flat_parts() below lists, for a sequence, which slots
// hold its partials; the merge kernel applies Equation 4 over them (over all KV holders of a
// ring at once, if asked to).
// ---------------------------------------------------------------------------
constexpr int FW = 4;                           // wavefronts per workgroup
constexpr int F_WG_PER_CU = 2;                  // (8 wavefronts per CU: 4 x 2 was faster than 8 x 1)
constexpr int FTHREADS = FW * 64;
constexpr int UNIT = 16;                        // keys per unit
constexpr int F_HALF_BYTES = UNIT * D * 2;      // K or V of one unit: 4 KiB
constexpr int F_POS_OFF = 2 * F_HALF_BYTES;     // kv_pos of the unit's keys, after K and V
constexpr int F_BUF_BYTES = F_POS_OFF + 256;    // one unit
constexpr int F_WAVE_LDS = 2 * F_BUF_BYTES;     // two units per wavefront
constexpr int F_SMEM = FW * F_WAVE_LDS;         // 66 KiB: two workgroups per CU
constexpr int F_UNIT_VMEM_OPS = 9;              // 4 K, 4 V and 1 position request per unit
static_assert(F_SMEM >= FW * CB_WAVE * 4, "combine buffer aliases the unit buffers");

struct FlatParams {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  const int32_t* q_pos;
  const int32_t* kv_pos;
  const int32_t* cu_kv;
  const int32_t* bid;
  float* part_out;   // [n_main + batch * FW][n_q_heads][D]
  float* part_lse;   // [n_main + batch * FW][n_q_heads]
  int32_t n_q;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t group;
  int32_t batch;
  int32_t total_kv;
  int32_t wg_keys;   // keys per workgroup range, a multiple of UNIT
  int32_t n_main;    // workgroups per KV head = main slots
  float scale_log2;
};

#define CP_LDS_AS __attribute__((address_space(3)))
#define CP_GLB_AS __attribute__((address_space(1)))
// 16 bytes per lane from global memory straight into LDS (lane l lands at dst + 16 l),
// non-temporal: K and V are read exactly once.
__device__ __forceinline__ void load_lds16_stream(const void* src, char* lds_dst_wave_uniform) {
  __builtin_amdgcn_global_load_lds((const CP_GLB_AS void*)src,
                                   (CP_LDS_AS void*)lds_dst_wave_uniform, 16, 0, 2);
}
typedef short shortx4_t __attribute__((ext_vector_type(4)));
// Waits until at most N vector-memory operations are outstanding; no memory access of the
// program moves across it.
template <int N>
__device__ __forceinline__ void vmem_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void lds_reads_done() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}
// LDS reads of a unit as inline assembly, waited for by hand: after a direct-to-LDS load the
// compiler puts a wait for ALL outstanding loads in front of every LDS read it knows about
// (it cannot tell the two unit buffers apart), which would serialise the two units in flight.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <int OFF>
__device__ __forceinline__ u32x4_t lds_read_b128_at(uint32_t addr) {
  u32x4_t r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// Transposed read: in a group of 16 lanes, lane i receives element i % 4 of the 8 bytes
// addressed by each of the lanes 4j + i / 4 (j = 0..3).
template <int OFF>
__device__ __forceinline__ u32x2_t lds_read_tr_at(uint32_t addr) {
  u32x2_t r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
template <int J>
struct IntC {
  static constexpr int value = J;
};

// max / sum of x over the lanes l, l ^ 16, l ^ 32, l ^ 48 (the four key sub-groups of a head),
// with lane-swap instructions on the vector pipe (no round trip through LDS). After
// v_permlane16_swap of two copies of x, the two registers hold x[l] and x[l ^ 16] in every
// lane, in some order; v_permlane32_swap likewise for l ^ 32. Inline assembly: through the
// builtins the compiler took the two results of a swap of equal operands for equal. (The
// s_nop covers the wait states a lane swap needs after a vector write of its operands.)
__device__ __forceinline__ void swap16(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap32(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float quad_max(float x) {
  float a = x, b = x;
  swap16(a, b);
  a = b = fmaxf(a, b);
  swap32(a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float quad_sum(float x) {
  float a = x, b = x;
  swap16(a, b);
  a = b = a + b;
  swap32(a, b);
  return a + b;
}

// What a wavefront knows of the sequence whose keys it is reading.
#define CP_INL __attribute__((always_inline))
struct SeqCtx {
  int s;            // sequence id
  int32_t lo, hi;   // its packed keys [lo, hi)
  int qi;           // its query, or -1
  int32_t qp;       // that query's position
  bf16x8_t qf[4];   // Q^T fragments: lane (hd, kg) holds channels kg*32 + ks*8 .. +7 of head hd
};

__global__ __launch_bounds__(FTHREADS, F_WG_PER_CU) void decode_flat_kernel(FlatParams p) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int hd = lane & 15;   // query head within the group (N side)
  const int kg = lane >> 4;   // key / channel sub-group
  const int g = blockIdx.x, kvh = blockIdx.y;
  const int32_t w0 = g * p.wg_keys;
  if (w0 >= p.total_kv) return;  // (no slot of such a workgroup is ever read)
  const int32_t w1 = min(w0 + p.wg_keys, p.total_kv);
  char* const buf0 = smem + wave * F_WAVE_LDS;
  char* const buf1 = buf0 + F_BUF_BYTES;

  // ---- unit requests: an instruction moves four rows (1 KiB); lane l covers row l / 16 of
  // the four and chunk position l % 16. Chunk c of K row r lands at position c ^ r, of V row
  // r at c ^ ((r & 3) * 4). Rows past the end of the range are clamped to its last row
  // (finite data; masked by their index). The unit's kv_pos travel the same way (lane l brings
  // the position of key l % 16): every operation of a unit is a request into LDS, none returns
  // a register, so the only waits are the counted ones below.
  const uint32_t tok_stride = (uint32_t)p.n_kv_heads * D;
  const int l_row = lane >> 4, l_pos = lane & 15;
  // per-lane element offsets of the eight requests of a full unit
  uint32_t koff[4], voff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = i * 4 + l_row;
    koff[i] = (uint32_t)row * tok_stride + ((l_pos ^ row) << 3);
    voff[i] = (uint32_t)row * tok_stride + ((l_pos ^ ((row & 3) << 2)) << 3);
  }
  auto issue_unit = [&](char* buf, int32_t key_req) CP_INL {
    // (a wavefront without a unit of its own still sends the requests, for the range's last
    // key: every wavefront then has the same number of operations in flight)
    const int32_t key0 = min(key_req, w1 - 1);
    const int last = min(UNIT, w1 - key0) - 1;
    const bf16_t* kt = p.k + (int64_t)key0 * tok_stride + kvh * D;
    const bf16_t* vt = p.v + (int64_t)key0 * tok_stride + kvh * D;
    if (__builtin_expect(last == UNIT - 1, 1)) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        load_lds16_stream(kt + koff[i], buf + i * 1024);
        load_lds16_stream(vt + voff[i], buf + F_HALF_BYTES + i * 1024);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = i * 4 + l_row;
        const uint32_t roff = (uint32_t)min(row, last) * tok_stride;
        load_lds16_stream(kt + roff + ((l_pos ^ row) << 3), buf + i * 1024);
        load_lds16_stream(vt + roff + ((l_pos ^ ((row & 3) << 2)) << 3),
                          buf + F_HALF_BYTES + i * 1024);
      }
    }
    __builtin_amdgcn_global_load_lds((const CP_GLB_AS void*)(p.kv_pos + key0 + min(l_pos, last)),
                                     (CP_LDS_AS void*)(buf + F_POS_OFF), 4, 0, 0);
  };

  // ---- who owns the keys: sequence s holds packed keys [cu[s], cu[s+1]) ----
  // The first 64 entries of cu_seqlens_kv (from index 1), bid and q_pos are requested one per
  // lane BEFORE the first units: vector loads return in issue order, so these are in the
  // registers after one short round trip while the units are still on their way, and every
  // lookup below is a ballot or a lane read. (Entries past 64 come through scalar loads, which
  // do not queue behind the units either.) The Q fragments depend on the lookups, so they
  // queue behind the first units and arrive with them; the sequence after the current one is
  // looked up, Q included, ahead of time, so that crossing into it costs no round trip behind
  // the units in flight.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_t;
  const const_i32_t cu_c = (const_i32_t)p.cu_kv, bid_c = (const_i32_t)p.bid,
                    qpos_c = (const_i32_t)p.q_pos;
  // (Inline assembly, waited for by hand below: the compiler, asked to wait for a load that
  // has direct-to-LDS loads behind it, waits for those as well.)
  int32_t t_cu, t_bid, t_qp;
  {
    const int32_t* a_cu = p.cu_kv + min(lane + 1, p.batch);
    const int32_t* a_bid = p.bid + min(lane, p.n_q - 1);
    const int32_t* a_qp = p.q_pos + min(lane, p.n_q - 1);
    asm volatile("global_load_dword %0, %3, off\n\t"
                 "global_load_dword %1, %4, off\n\t"
                 "global_load_dword %2, %5, off"
                 : "=&v"(t_cu), "=&v"(t_bid), "=&v"(t_qp)
                 : "v"(a_cu), "v"(a_bid), "v"(a_qp)
                 : "memory");
  }

  int32_t key_a = w0 + wave * UNIT;        // unit in buf0
  int32_t key_b = key_a + FW * UNIT;       // unit in buf1
  issue_unit(buf0, key_a);
  issue_unit(buf1, key_b);
  // the three table loads precede the 2 * F_UNIT_VMEM_OPS operations of the two units
  asm volatile("s_waitcnt vmcnt(%3)"
               : "+v"(t_cu), "+v"(t_bid), "+v"(t_qp)
               : "n"(2 * F_UNIT_VMEM_OPS));

  const bool head_ok = hd < p.group;
  auto cu_at = [&](int i) CP_INL -> int32_t {  // cu_seqlens_kv[i], i wave-uniform
    if (i == 0) return 0;
    return i <= 64 ? __builtin_amdgcn_readlane(t_cu, i - 1) : cu_c[i];
  };
  auto lookup = [&](SeqCtx& c, int s) CP_INL {  // s is wave-uniform, 0 <= s < batch
    c.s = s;
    c.lo = cu_at(s);
    c.hi = cu_at(s + 1);
    // the query of this sequence: the first i with bid[i] == s, or none
    const uint64_t hit = __builtin_amdgcn_ballot_w64(lane < p.n_q && t_bid == s);
    c.qi = hit != 0 ? (int)__builtin_ctzll(hit) : -1;
    const int last_q = p.n_q - 1;
    for (int i = 64; i <= last_q && c.qi < 0; i += 4) {
      const int i1 = min(i + 1, last_q), i2 = min(i + 2, last_q), i3 = min(i + 3, last_q);
      const int b0 = bid_c[i], b1 = bid_c[i1], b2 = bid_c[i2], b3 = bid_c[i3];
      c.qi = b0 == s ? i : b1 == s ? i1 : b2 == s ? i2 : b3 == s ? i3 : -1;
    }
    c.qp = c.qi < 0 ? CP_POS_PAD_Q
                    : c.qi < 64 ? __builtin_amdgcn_readlane(t_qp, c.qi) : qpos_c[c.qi];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 t = make_uint4(0, 0, 0, 0);
      if (c.qi >= 0 && head_ok)
        t = *(const uint4*)(p.q + ((int64_t)c.qi * p.n_q_heads + kvh * p.group + hd) * D +
                            kg * 32 + ks * 8);
      c.qf[ks] = __builtin_bit_cast(bf16x8_t, t);
    }
    // The fragments are needed in registers now: the compiler waits for them here, once, and
    // not (for want of an exact count) for everything in flight at every later use. At the
    // start that wait is the first units' own; after that it is only reached when a third
    // sequence begins inside the range.
    asm volatile("" ::"v"(c.qf[0]), "v"(c.qf[1]), "v"(c.qf[2]), "v"(c.qf[3]));
  };
  SeqCtx cur, nxt;
  bool have_next = false;
  {
    // the largest s with cu[s] <= w0: the number of i in [1, batch) with cu[i] <= w0
    const int in_table = min(64, p.batch - 1);
    int lo = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane < in_table && t_cu <= w0));
    if (lo == 64 && p.batch - 1 > 64) {  // beyond the table: bisection with scalar loads
      int hi = p.batch - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (cu_c[mid] <= w0) lo = mid;
        else hi = mid - 1;
      }
    }
    lookup(cur, lo);
  }
  // Looks ahead to the sequence after `cur` if it begins inside the range.
  auto look_ahead = [&]() CP_INL {
    have_next = cur.hi < w1 && cur.s + 1 < p.batch;
    if (have_next) lookup(nxt, cur.s + 1);
  };
  look_ahead();

  float m_run = -INFINITY, l_run = 0.f;
  floatx4_t o_acc[8];
  auto reset_state = [&]() CP_INL {
    m_run = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) o_acc[db] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  };
  reset_state();

  // This wavefront's partial of the sequence that ends inside the range: normalised O and LSE
  // to the sequence's tail slot of this wavefront (LSE only when it saw nothing).
  auto flush_tail = [&]() CP_INL {
    if (cur.qi >= 0 && cur.hi > cur.lo) {
      const float l_tot = quad_sum(l_run);
      const int64_t slot = (int64_t)p.n_main + (int64_t)cur.s * FW + wave;
      const int64_t row = slot * p.n_q_heads + kvh * p.group + hd;
      if (head_ok) {
        if (l_tot > 0.f) {
          const float inv = 1.f / l_tot;
#pragma unroll
          for (int db = 0; db < 8; ++db) {
            floatx4_t w = {o_acc[db][0] * inv, o_acc[db][1] * inv, o_acc[db][2] * inv,
                           o_acc[db][3] * inv};
            *(floatx4_t*)(p.part_out + row * D + db * 16 + kg * 4) = w;
          }
        }
        if (kg == 0)
          p.part_lse[row] =
              l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      }
    }
    reset_state();
  };
  // Moves on to the next sequence; false when there is none (then cu_seqlens_kv does not end
  // at total_kv: nothing more is read).
  auto next_seq = [&]() CP_INL -> bool {
    if (!have_next) return false;
    cur = nxt;
    look_ahead();
    return true;
  };

  // ---- fragment addresses (LDS byte addresses inside the unit buffer 0 of this wavefront) ----
  const uint32_t lds_base = (uint32_t)(size_t)(CP_LDS_AS char*)smem + wave * F_WAVE_LDS;
  // K: A-operand row of this lane is key hd; its channels kg*32 + ks*8 .. +7 are chunk kg*4 + ks
  uint32_t kaddr[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) kaddr[ks] = lds_base + hd * 256 + (((kg * 4 + ks) ^ hd) << 4);
  // V^T: in its group of 16 lanes this lane addresses key kg*4 + vj and the 8 bytes (4 channels)
  // vq of the 16-channel strip of block db
  uint32_t vaddr[8];
  {
    const int vj = (lane & 15) >> 2, vq = lane & 3;
    const int r = kg * 4 + vj;
#pragma unroll
    for (int db = 0; db < 8; ++db)
      vaddr[db] = lds_base + F_HALF_BYTES + r * 256 + (vq & 1) * 8 +
                  (((db * 2 + (vq >> 1)) ^ ((r & 3) << 2)) << 4);
  }
  const uint32_t paddr = lds_base + F_POS_OFF + kg * 16;  // kv_pos of the keys kg*4 + i

  // S^T and O^T of the keys [lo, hi) of the unit at t0 (in unit buffer BUF) for the current
  // sequence
  auto unit_compute = [&](auto bufc, int32_t t0, int32_t lo, int32_t hi) CP_INL {
    constexpr int BO = decltype(bufc)::value * F_BUF_BYTES;
    u32x4_t kp4 = lds_read_b128_at<BO>(paddr);
    u32x4_t kf0 = lds_read_b128_at<BO>(kaddr[0]), kf1 = lds_read_b128_at<BO>(kaddr[1]);
    u32x4_t kf2 = lds_read_b128_at<BO>(kaddr[2]), kf3 = lds_read_b128_at<BO>(kaddr[3]);
    u32x2_t vf0 = lds_read_tr_at<BO>(vaddr[0]), vf1 = lds_read_tr_at<BO>(vaddr[1]);
    u32x2_t vf2 = lds_read_tr_at<BO>(vaddr[2]), vf3 = lds_read_tr_at<BO>(vaddr[3]);
    u32x2_t vf4 = lds_read_tr_at<BO>(vaddr[4]), vf5 = lds_read_tr_at<BO>(vaddr[5]);
    u32x2_t vf6 = lds_read_tr_at<BO>(vaddr[6]), vf7 = lds_read_tr_at<BO>(vaddr[7]);
    // the K fragments and positions are there once at most the 8 V reads are outstanding
    asm volatile("s_waitcnt lgkmcnt(8)"
                 : "+v"(kp4), "+v"(kf0), "+v"(kf1), "+v"(kf2), "+v"(kf3));
    floatx4_t s = {0.f, 0.f, 0.f, 0.f};
    s = mfma16(__builtin_bit_cast(bf16x8_t, kf0), cur.qf[0], s);
    s = mfma16(__builtin_bit_cast(bf16x8_t, kf1), cur.qf[1], s);
    s = mfma16(__builtin_bit_cast(bf16x8_t, kf2), cur.qf[2], s);
    s = mfma16(__builtin_bit_cast(bf16x8_t, kf3), cur.qf[3], s);
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // (lo <= key index < hi as one unsigned comparison)
      const uint32_t off = (uint32_t)(t0 + kg * 4 + i - lo);
      if ((int32_t)kp4[i] > cur.qp || off >= (uint32_t)(hi - lo)) s[i] = -INFINITY;
      mx = fmaxf(mx, s[i]);
    }
    mx = quad_max(mx);
    const float m_new = fmaxf(m_run, mx * p.scale_log2);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    float lsum = 0.f;
    bf16x4_t pb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float e = __builtin_amdgcn_exp2f(fmaf(s[i], p.scale_log2, -m_use));
      lsum += e;
      pb[i] = static_cast<bf16_t>(e);
    }
    l_run = fmaf(l_run, alpha, lsum);
    m_run = m_new;
    // O^T += V^T P^T over 8 blocks of 16 channels; slot i of this lane's P^T slice is key
    // kg*4 + i, which is what the transposed reads fetched for this lane's channel
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(vf0), "+v"(vf1), "+v"(vf2), "+v"(vf3), "+v"(vf4), "+v"(vf5), "+v"(vf6),
                   "+v"(vf7));
    const u32x2_t vf[8] = {vf0, vf1, vf2, vf3, vf4, vf5, vf6, vf7};
    const shortx4_t pb4 = __builtin_bit_cast(shortx4_t, pb);
    // the running maximum of a head rarely moves after its first units: rescale only then
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
      for (int db = 0; db < 8; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) o_acc[db][i] *= alpha;
    }
#pragma unroll
    for (int db = 0; db < 8; ++db)
      o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
          __builtin_bit_cast(shortx4_t, vf[db]), pb4, o_acc[db], 0, 0, 0);
  };

  // One unit, whichever sequences it holds. `more` turns false when the sequences run out.
  bool more = true;
  auto process_unit = [&](auto bufc, int32_t key0) CP_INL {
    const int32_t t1 = min(key0 + UNIT, w1);
    // (one call site for the products: two would make the compiler shuttle the accumulators
    // between register sets at every unit)
    while (more) {
      if (__builtin_expect(cur.hi <= key0, 0)) {  // a sequence that ended before this unit
        flush_tail();
        more = next_seq();
        continue;
      }
      if (cur.qi >= 0) unit_compute(bufc, key0, max(cur.lo, key0), min(cur.hi, t1));
      if (__builtin_expect(cur.hi >= t1, 1)) break;
      flush_tail();  // the sequence ends inside this unit
      more = next_seq();
    }
  };

  while (key_a < w1) {
    // the unit in buf0 has landed once only the later unit's operations are outstanding
    if (key_b < w1) vmem_wait<F_UNIT_VMEM_OPS>();
    else vmem_wait<0>();
    process_unit(IntC<0>{}, key_a);
    lds_reads_done();  // before the buffer is refilled
    key_a = key_b + FW * UNIT;
    if (key_a < w1) issue_unit(buf0, key_a);
    if (key_b >= w1) break;
    if (key_a < w1) vmem_wait<F_UNIT_VMEM_OPS>();
    else vmem_wait<0>();
    process_unit(IntC<1>{}, key_b);
    lds_reads_done();
    key_b = key_a + FW * UNIT;
    if (key_b < w1) issue_unit(buf1, key_b);
  }
  // sequences that end inside the range after this wavefront's last unit
  while (more && cur.hi < w1) {
    flush_tail();
    more = next_seq();
  }

  // ---- combine the wavefronts (disjoint key subsets of one sequence) in LDS ----
  l_run = quad_sum(l_run);
  __syncthreads();  // all unit buffers are dead
  float* const cbuf = (float*)smem;
  float* const my = cbuf + wave * CB_WAVE;
  // accumulator (db, i) of lane (hd, kg) is channel db*16 + kg*4 + i
#pragma unroll
  for (int db = 0; db < 8; ++db) *(floatx4_t*)(my + hd * CB_STRIDE + db * 16 + kg * 4) = o_acc[db];
  if (kg == 0) {
    my[16 * CB_STRIDE + hd] = m_run;
    my[16 * CB_STRIDE + 16 + hd] = l_run;
  }
  __syncthreads();
  // thread -> (head, CPT consecutive channels)
  {
    constexpr int CPT = 16 * D / FTHREADS, TPH = D / CPT;
    const int h = tid / TPH, d0 = (tid % TPH) * CPT;
    float mw[FW], lw[FW], mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < FW; ++w) {
      mw[w] = cbuf[w * CB_WAVE + 16 * CB_STRIDE + h];
      lw[w] = cbuf[w * CB_WAVE + 16 * CB_STRIDE + 16 + h];
      mmax = fmaxf(mmax, mw[w]);
    }
    floatx4_t acc[CPT / 4];
#pragma unroll
    for (int c = 0; c < CPT / 4; ++c) acc[c] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    if (mmax != -INFINITY) {
#pragma unroll
      for (int w = 0; w < FW; ++w) {
        const float f = __builtin_amdgcn_exp2f(mw[w] - mmax);
        den = fmaf(lw[w], f, den);
        const float* src = cbuf + w * CB_WAVE + h * CB_STRIDE + d0;
#pragma unroll
        for (int c = 0; c < CPT / 4; ++c) {
          const floatx4_t x = *(const floatx4_t*)(src + 4 * c);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[c][e] = fmaf(x[e], f, acc[c][e]);
        }
      }
    }
    if (h < p.group) {
      const int64_t row = (int64_t)g * p.n_q_heads + kvh * p.group + h;
      const float inv = den > 0.f ? 1.f / den : 0.f;
      float* o = p.part_out + row * D + d0;
#pragma unroll
      for (int c = 0; c < CPT / 4; ++c) {
        floatx4_t v = {acc[c][0] * inv, acc[c][1] * inv, acc[c][2] * inv, acc[c][3] * inv};
        *(floatx4_t*)(o + 4 * c) = v;
      }
      if (tid % TPH == 0)
        p.part_lse[row] = den > 0.f ? (mmax + __builtin_amdgcn_logf(den)) * kLn2 : -INFINITY;
    }
  }
}

// Which slots hold the partials of sequence [a, b) of a rank whose ranges are wg_keys long:
// main slots g_lo .. g_hi (the workgroups whose range ends inside the sequence, or at its
// end), and, if the sequence ends strictly inside a range, the FW tail slots of that sequence.
struct FlatParts {
  int g_lo, g_hi;  // empty when g_hi < g_lo
  bool tail;
};
__host__ __device__ inline FlatParts flat_parts(int32_t a, int32_t b, int32_t wg_keys,
                                                int32_t total_kv) {
  FlatParts r;
  r.g_lo = 0; r.g_hi = -1; r.tail = false;
  if (b <= a) return r;
  r.g_lo = a / wg_keys;
  r.g_hi = b >= total_kv ? (total_kv + wg_keys - 1) / wg_keys - 1 : b / wg_keys - 1;
  r.tail = b < total_kv && b % wg_keys != 0;
  return r;
}

// Equation 4 over the flat decode partials of one query row (query, head), over all holders.
// One workgroup of MW wavefronts per row. Thread t looks up part t of the row (its slot and
// LSE); the largest LSE and the weights are reduced across the workgroup; then the wavefronts
// share out the parts, every lane accumulating two channels of the parts its wavefront takes
// (four loads in flight per lane), and the MW sums are added up in LDS.
constexpr int kMaxHolders = CP_MAX_PARTS;
struct FlatMergeParams {
  const float* part_out[kMaxHolders];
  const float* part_lse[kMaxHolders];
  const int32_t* cu_kv[kMaxHolders];
  int32_t total_kv[kMaxHolders];
  int32_t wg_keys[kMaxHolders];
  int32_t n_main[kMaxHolders];
  const int32_t* bid;
  int32_t n_holders;
  int32_t n_q_heads;
};

// MW wavefronts per workgroup: 16 for a ring of holders, 4 for the few parts of one call
// (measured: 2 -> 4 wavefronts 6.0 -> 5.3 us; eight loads in flight per lane instead of four
// gain nothing there and cost the ring's merge 6 %).
constexpr int FM_U = 4;     // row loads in flight per lane
constexpr int FM_MW1 = 4;   // wavefronts per row for one holder
template <typename TO, int MW>
__global__ __launch_bounds__(MW * 64) void decode_flat_merge_kernel(FlatMergeParams mp,
                                                                     TO* __restrict__ out,
                                                                     float* __restrict__ lse_out) {
  constexpr int MTHREADS = MW * 64;
  static_assert(MTHREADS >= D, "one thread per channel writes the row");
  __shared__ int part_begin[kMaxHolders + 1];  // first part index of every holder
  __shared__ int holder_lo[kMaxHolders], holder_mains[kMaxHolders];
  __shared__ float red[MW];
  __shared__ float w_of[MTHREADS];
  __shared__ const float* src_of[MTHREADS];
  __shared__ float sums[MW][D];
  const int row = blockIdx.x;  // query * n_q_heads + head
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int qi = row / mp.n_q_heads, h = row - qi * mp.n_q_heads;
  const int s = mp.bid[qi];
  // thread k looks up holder k's slots of this sequence (one round trip for all holders),
  // thread 0 then lines the holders' parts up
  if (tid < mp.n_holders) {
    const int k = tid;
    const FlatParts fp =
        flat_parts(mp.cu_kv[k][s], mp.cu_kv[k][s + 1], mp.wg_keys[k], mp.total_kv[k]);
    const int mains = max(0, fp.g_hi - fp.g_lo + 1);
    holder_lo[k] = fp.g_lo;
    holder_mains[k] = mains;
    part_begin[k + 1] = mains + (fp.tail ? FW : 0);
  }
  __syncthreads();
  if (tid == 0) {
    int n = 0;
    for (int k = 0; k < mp.n_holders; ++k) {
      const int c = part_begin[k + 1];
      part_begin[k] = n;
      n += c;
    }
    part_begin[mp.n_holders] = n;
  }
  __syncthreads();
  const int n_parts = part_begin[mp.n_holders];
  float acc0 = 0.f, acc1 = 0.f, den = 0.f, lmax = -INFINITY;
  // (more than MTHREADS parts: several passes, each merged into the running result)
  for (int base = 0; base < n_parts; base += MTHREADS) {
    const int t = base + tid;
    float my_lse = -INFINITY;
    const float* my_src = nullptr;
    if (t < n_parts) {
      int k = 0;
      while (part_begin[k + 1] <= t) ++k;
      const int j = t - part_begin[k];
      const int64_t slot = j < holder_mains[k]
                               ? (int64_t)holder_lo[k] + j
                               : (int64_t)mp.n_main[k] + (int64_t)s * FW + (j - holder_mains[k]);
      my_lse = mp.part_lse[k][slot * mp.n_q_heads + h];
      my_src = mp.part_out[k] + (slot * mp.n_q_heads + h) * D;
    }
    float pmax = my_lse;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) pmax = fmaxf(pmax, __shfl_xor(pmax, o, 64));
    if (lane == 0) red[wave] = pmax;
    __syncthreads();
    pmax = red[0];
#pragma unroll
    for (int w = 1; w < MW; ++w) pmax = fmaxf(pmax, red[w]);
    const float new_max = fmaxf(lmax, pmax);
    if (new_max != -INFINITY) {  // uniform
      const float rescale = __expf(lmax - new_max);  // 0 on the first pass with data
      acc0 *= rescale;
      acc1 *= rescale;
      den *= rescale;
      lmax = new_max;
      const float w = __expf(my_lse - lmax);  // exp(-inf) = 0: an empty part
      w_of[tid] = w;
      src_of[tid] = my_src;
      float wsum = w;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) wsum += __shfl_xor(wsum, o, 64);
      __syncthreads();  // red[] fully read; w_of / src_of visible
      if (lane == 0) red[wave] = wsum;
      const int cnt = min(MTHREADS, n_parts - base);
      for (int e = wave; e < cnt; e += FM_U * MW) {
        typedef float floatx2_t __attribute__((ext_vector_type(2)));
        float wj[FM_U];
        floatx2_t x[FM_U];
#pragma unroll
        for (int u = 0; u < FM_U; ++u) {
          const int ee = min(e + u * MW, cnt - 1);
          wj[u] = e + u * MW < cnt ? w_of[ee] : 0.f;
          // a part with zero weight may hold anything (it is read, then dropped)
          x[u] = __builtin_nontemporal_load((const floatx2_t*)src_of[ee] + lane);
        }
#pragma unroll
        for (int u = 0; u < FM_U; ++u) {
          acc0 = fmaf(wj[u], wj[u] != 0.f ? x[u][0] : 0.f, acc0);
          acc1 = fmaf(wj[u], wj[u] != 0.f ? x[u][1] : 0.f, acc1);
        }
      }
      __syncthreads();
      float dsum = red[0];
#pragma unroll
      for (int w2 = 1; w2 < MW; ++w2) dsum += red[w2];
      den += dsum;
    }
    __syncthreads();
  }
  sums[wave][lane * 2] = acc0;
  sums[wave][lane * 2 + 1] = acc1;
  __syncthreads();
  if (tid < D) {
    float r = 0.f;
#pragma unroll
    for (int w = 0; w < MW; ++w) r += sums[w][tid];
    out[(int64_t)row * D + tid] = from_float<TO>(den > 0.f ? r / den : 0.f);
  }
  if (lse_out != nullptr && tid == 0) lse_out[row] = den > 0.f ? lmax + __logf(den) : -INFINITY;
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

// ---- flat path: plan, launches ----
bool decode_flat_applies(const cp_shape& s) {
  // the caller's promise that no sequence id occurs twice; and most sequences have a query
  // (the flat ranges read every key of the rank, wanted or not)
  return (s.flags & CP_SHAPE_UNIQUE_BID) != 0 && s.total_q > 0 && s.total_kv > 0 &&
         2 * s.total_q >= s.batch && s.total_q <= 0x3fffffff;
}

namespace {
struct FlatPlan {
  int n_main, wg_keys;
  size_t slots, out_bytes, lse_bytes;
};
FlatPlan flat_plan(const cp_shape& s) {
  FlatPlan pl;
  pl.n_main = std::max(1, 256 * F_WG_PER_CU / s.n_kv_heads);  // all resident, over all KV heads
  const int64_t per = (s.total_kv + pl.n_main - 1) / pl.n_main;
  pl.wg_keys = (int)std::max<int64_t>(UNIT, (per + UNIT - 1) / UNIT * UNIT);
  pl.slots = (size_t)pl.n_main + (size_t)s.batch * FW;
  pl.out_bytes = round256(pl.slots * s.n_q_heads * D * 4);
  pl.lse_bytes = round256(pl.slots * s.n_q_heads * 4);
  return pl;
}
}  // namespace

size_t decode_flat_region_bytes(const cp_shape& s) {
  const FlatPlan pl = flat_plan(s);
  return pl.out_bytes + pl.lse_bytes;
}

int launch_decode_flat_partials(const cp_shape& s, float scale, const void* q, const void* k,
                                const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                                const int32_t* cu_kv, const int32_t* bid, void* region,
                                size_t region_bytes, hipStream_t stream) {
  const FlatPlan pl = flat_plan(s);
  if (region_bytes < pl.out_bytes + pl.lse_bytes) return CP_ERR_WORKSPACE;
  if (s.n_kv_heads > 65535) return CP_ERR_SHAPE;
  // key indices, range starts and per-lane offsets inside a tile are kept in 32 bits
  if (s.total_kv > 0x7fffffffLL - 2 * (int64_t)pl.wg_keys) return CP_ERR_SHAPE;
  if ((int64_t)s.n_kv_heads * D * 64 > 0x7fffffffLL) return CP_ERR_SHAPE;
  FlatParams p;
  p.q = (const bf16_t*)q; p.k = (const bf16_t*)k; p.v = (const bf16_t*)v;
  p.q_pos = q_pos; p.kv_pos = kv_pos; p.cu_kv = cu_kv; p.bid = bid;
  p.part_out = (float*)region;
  p.part_lse = (float*)((char*)region + pl.out_bytes);
  p.n_q = (int32_t)s.total_q;
  p.n_q_heads = s.n_q_heads; p.n_kv_heads = s.n_kv_heads;
  p.group = s.n_q_heads / s.n_kv_heads;
  p.batch = s.batch;
  p.total_kv = (int32_t)s.total_kv;
  p.wg_keys = pl.wg_keys;
  p.n_main = pl.n_main;
  p.scale_log2 = scale * kLog2e;
  if (hipFuncSetAttribute((const void*)decode_flat_kernel,
                          hipFuncAttributeMaxDynamicSharedMemorySize, F_SMEM) != hipSuccess)
    return CP_ERR_LAUNCH;
  hipLaunchKernelGGL(decode_flat_kernel, dim3(pl.n_main, s.n_kv_heads), dim3(FTHREADS), F_SMEM,
                     stream, p);
  return check_launch();
}

int launch_decode_flat_merge(int n_holders, const cp_shape* shapes, void* const* regions,
                             const int32_t* const* cu_kv, const int32_t* bid, int64_t n_q,
                             void* out, int32_t out_dtype, float* lse, hipStream_t stream) {
  if (n_holders < 1 || n_holders > kMaxHolders) return CP_ERR_SHAPE;
  if (n_q == 0) return CP_OK;
  FlatMergeParams mp = {};
  for (int k = 0; k < n_holders; ++k) {
    const FlatPlan pl = flat_plan(shapes[k]);
    mp.part_out[k] = (const float*)regions[k];
    mp.part_lse[k] = (const float*)((const char*)regions[k] + pl.out_bytes);
    mp.cu_kv[k] = cu_kv[k];
    mp.total_kv[k] = (int32_t)shapes[k].total_kv;
    mp.wg_keys[k] = pl.wg_keys;
    mp.n_main[k] = pl.n_main;
  }
  mp.bid = bid;
  mp.n_holders = n_holders;
  mp.n_q_heads = shapes[0].n_q_heads;
  const int64_t rows = n_q * shapes[0].n_q_heads;
  if (rows > 0x7fffffffLL) return CP_ERR_SHAPE;
  const dim3 grid((unsigned)rows);
  if (n_holders == 1) {
    if (out_dtype == CP_FP32)
      hipLaunchKernelGGL((decode_flat_merge_kernel<float, FM_MW1>), grid, dim3(FM_MW1 * 64), 0, stream, mp,
                         (float*)out, lse);
    else
      hipLaunchKernelGGL((decode_flat_merge_kernel<bf16_t, FM_MW1>), grid, dim3(FM_MW1 * 64), 0, stream, mp,
                         (bf16_t*)out, lse);
  } else {
    if (out_dtype == CP_FP32)
      hipLaunchKernelGGL((decode_flat_merge_kernel<float, 16>), grid, dim3(1024), 0, stream, mp,
                         (float*)out, lse);
    else
      hipLaunchKernelGGL((decode_flat_merge_kernel<bf16_t, 16>), grid, dim3(1024), 0, stream, mp,
                         (bf16_t*)out, lse);
  }
  return check_launch();
}

size_t decode_workspace_bytes(const cp_shape& s) {
  if (decode_flat_applies(s)) return decode_flat_region_bytes(s);
  const int splits = plan_splits(s);
  const size_t rows = (size_t)s.total_q * s.n_q_heads;
  return round256(splits * rows * D * 4) + round256(splits * rows * 4);
}

int launch_decode(const cp_shape& s, float scale, const void* q, const void* k, const void* v,
                  const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_kv,
                  const int32_t* bid, void* out, float* lse, int32_t out_dtype, void* workspace,
                  size_t workspace_bytes, hipStream_t stream) {
  if (decode_flat_applies(s)) {
    const int rc = launch_decode_flat_partials(s, scale, q, k, v, q_pos, kv_pos, cu_kv, bid,
                                               workspace, workspace_bytes, stream);
    if (rc != CP_OK) return rc;
    return launch_decode_flat_merge(1, &s, &workspace, &cu_kv, bid, s.total_q, out, out_dtype, lse,
                                    stream);
  }
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

