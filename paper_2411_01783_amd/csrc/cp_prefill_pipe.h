// Software-pipelined bf16 MFMA partial-attention kernel (included by cp_prefill_mfma.hip,
// which defines Params, the tile constants and the LDS layout used here).
//
// K and V tiles travel HBM/L2 -> LDS with global_load_lds (16 bytes per lane, no register
// staging): both are stored row-major [key][256 B]; bank conflicts are avoided by permuting
// the 16-byte chunks of a row on the GLOBAL side (chunk c of K row r lands at position
// c ^ (r & 15), chunk c of V row r at c ^ ((r & 3) * 4)). K fragments (rows = keys) are
// read with ds_read_b128, V^T fragments (rows = channels) with ds_read_b64_tr_b16.
//
// The KV axis is consumed in blocks of 32 keys and each wavefront runs three stages at
// once, one block apart:
//     P(i-1):  O^T += V^T P^T of the previous block        (8 MFMA, matrix pipe)
//     SM(i):   mask, row maximum, exponentials of block i   (vector pipe)
//     Q(i+1):  S^T = K Q^T of the next block                (8 MFMA, matrix pipe)
// The three are independent, so the vector work is issued between the MFMAs of its
// neighbours, one slice per MFMA, in source order (scheduling fences keep that order).
// LDS fragment reads are inline assembly with hand-counted lgkmcnt waits, issued eight
// MFMAs before their use: the compiler would otherwise wait for the tile prefetch
// (vmcnt(0)) in front of every LDS read that follows a direct-to-LDS load, and would not
// keep reads in flight across its own waits.
//
// Synchronisation per 128-key tile, two buffers: barrier Y before the last block of a tile
// (the next tile has landed; that block's Q stage reads its first 32 keys), barrier X after
// it (every read of the current tile has completed; the tile after the next is requested
// into its buffer).
#pragma once

#define CP_LDS_AS __attribute__((address_space(3)))
#define CP_GLB_AS __attribute__((address_space(1)))

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

constexpr int ROW_BYTES = D * 2;              // one K or V row in LDS
constexpr int KD_BYTES = TILE * ROW_BYTES;    // 32 KiB per tile buffer
constexpr int BLK_BYTES = 32 * ROW_BYTES;     // one 32-key block of a tile
constexpr int OFF_V8 = 2 * KD_BYTES;
constexpr int OFF_POS8 = OFF_V8 + 2 * KD_BYTES;
constexpr int OFF_SCRATCH8 = OFF_POS8 + 2 * POS_BYTES;
constexpr int OFF_LIVE8 = OFF_SCRATCH8 + 128;
constexpr int SMEM_BYTES8 = OFF_LIVE8 + MAX_LIVE * 16;
static_assert(NWAVE * 32 * OUT_STRIDE <= SMEM_BYTES8, "epilogue staging fits in the allocation");
static_assert(SMEM_BYTES8 <= 160 * 1024, "LDS budget of one CU");
static_assert(2 * KD_BYTES <= 65536, "K fragment offsets fit the 16-bit LDS offset field");

__device__ __forceinline__ void load_lds16(const void* src, char* lds_dst_wave_uniform) {
  __builtin_amdgcn_global_load_lds((const CP_GLB_AS void*)src, (CP_LDS_AS void*)lds_dst_wave_uniform,
                                   16, 0, 0);
}

template <int OFF>
__device__ __forceinline__ u32x4_t lds_read_b128(uint32_t addr) {
  u32x4_t r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// Lane i of a 16-lane group receives element i % 4 of the 8 bytes addressed by each of the
// lanes 4j + i / 4 (j = 0..3) of the group: four lanes address four consecutive keys of a
// 16-channel strip and every lane receives one channel of those four keys.
template <int OFF>
__device__ __forceinline__ u32x2_t lds_read_tr(uint32_t addr) {
  u32x2_t r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// Wait until at most N LDS operations issued after the one that fills the operands are
// outstanding. The operands are tied to the statement so that their consumer cannot be
// scheduled above the wait.
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x4_t& x) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N < 15 ? N : 15));
}
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x2_t& x, u32x2_t& y) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(N < 15 ? N : 15));
}
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x4_t& a, u32x4_t& b, u32x4_t& c, u32x4_t& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)"
               : "+v"(a), "+v"(b), "+v"(c), "+v"(d)
               : "n"(N < 15 ? N : 15));
}
// A V^T fragment is two transposed reads into the halves of one 128-bit register tuple.
template <int OFF>
__device__ __forceinline__ u32x4_t lds_read_vt_frag(uint32_t addr) {
  const u32x2_t lo = lds_read_tr<OFF>(addr), hi = lds_read_tr<OFF + 8 * ROW_BYTES>(addr);
  const u32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
  return v;
}
// Keeps the computation of x at this point of the instruction stream (the optimiser would
// otherwise sink the softmax arithmetic to its first use, one pipeline step later).
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(unsigned& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  bf16x2_t t;
  t[0] = static_cast<bf16_t>(a);
  t[1] = static_cast<bf16_t>(b);
  return __builtin_bit_cast(unsigned, t);
}

// Workgroup barrier that orders LDS traffic only: global loads issued before it (the Q
// fragments, the tile-bound prefetch) stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Everything a wavefront carries from block to block. All indices are compile-time.
struct PipeRegs {
  floatx16_t o[4];         // O^T accumulators, 4 blocks of 32 channels
  floatx16_t s[2];         // scores of block i (index: parity of i) and of block i+1
  u32x4_t pb[2][2];        // probabilities (bf16 pairs) of block i (parity of i) / i-1, two 16-key slices
  u32x4_t kf[8];           // K fragments of block i+1
  u32x4_t vf[8];           // V^T fragments of block i-1
  float m_run, l_run;
};


template <int J>
struct IntC {
  static constexpr int value = J;
};

// One pipeline step for block BLK of the current tile. kaddr / vaddr / paddr are this
// lane's LDS byte addresses into the K buffer that holds block BLK+1, the V buffer of the
// current tile and its kv_pos.
// Accumulator idx of S^T in lane (n, g) is key (idx/4)*8 + g*4 + idx%4 of the block and query
// n; slot jj of the lane's slice of P^T in MFMA kk is key kk*16 + (jj/4)*8 + g*4 + jj%4,
// which is the order in which the V^T fragments are fetched.
// `hook(IntC<M>)` runs after MFMA M (0..15) of the step: the caller spreads the requests
// for the next tile over these points, a different one for every wavefront, so that no
// wavefront queues behind a burst of loads.
template <int BLK, bool BAND, typename Hook>
__device__ __forceinline__ void pipe_body(PipeRegs& R, const bf16x8_t (&qf)[8],
                                          const uint32_t (&kaddr)[8], const uint32_t (&vaddr)[4],
                                          uint32_t paddr, int32_t qp, int32_t ql,
                                          float scale_log2, bool need_mask, bool& have_ref,
                                          Hook hook) {
  constexpr int CUR = BLK & 1, NXT = CUR ^ 1;
  constexpr int KOFF = ((BLK + 1) & 3) * BLK_BYTES;
  constexpr int VOFF = BLK * BLK_BYTES;
  constexpr int POFF = BLK * 32 * 4;
  // exponentials started by vector slice 1 + k: values [kBound[k], kBound[k + 1]); they are
  // summed and packed one slice later (a transcendental result has a wait state)
  constexpr int kBound[15] = {0, 1, 2, 3, 5, 6, 7, 8, 9, 10, 11, 13, 14, 15, 16};

  floatx16_t& s = R.s[CUR];
  float e[16];
  float m_use = 0.f, alpha = 1.f;
  float lsum0 = 0.f, lsum1 = 0.f;
  bool raise = false;

  // Online softmax in the log2 domain, reference maximum m_run per row.
  // Full form (masked tiles, and until every row of the wavefront has a reference): block
  // maximum, and the reference is raised when the maximum exceeds it by more than
  // kRescaleSlack. Fast form (everything else): no maximum at all. The exponentials are taken
  // against the standing reference, whatever the block holds; the reference is never above a
  // score the row has seen, so nothing underflows that should not, and a block whose
  // exponentials sum to more than kOverflowSum (a score 40 log2 units above the reference) is
  // detected from its sum and redone in the full form. O and l are rescaled at the end of
  // the step, after the MFMAs that still belong to the old reference. The denominator sums
  // the unrounded exponentials: LSE must be good to 1e-3 even on rows with a handful of
  // keys, which bf16 rounding of P would not give.
  auto block_max = [&]() __attribute__((always_inline)) -> float {
    float a = fmaxf(fmaxf(s[0], s[1]), s[2]);
    float b = fmaxf(fmaxf(s[3], s[4]), s[5]);
    float c = fmaxf(fmaxf(s[6], s[7]), s[8]);
    float d = fmaxf(fmaxf(s[9], s[10]), s[11]);
    a = fmaxf(fmaxf(a, s[12]), s[13]);
    b = fmaxf(fmaxf(b, s[14]), s[15]);
    const float mx = fmaxf(fmaxf(a, b), fmaxf(c, d));
    return fmaxf(mx, xor32(mx));
  };
  auto finish = [&](int v) __attribute__((always_inline)) {
    if (v & 1) {
      lsum1 += e[v];
      unsigned pk = pack_bf16(e[v - 1], e[v]);
      pin(pk);
      pin(lsum1);
      R.pb[CUR][v >> 3][(v & 7) >> 1] = pk;
    } else {
      lsum0 += e[v];
      pin(lsum0);
    }
  };

  auto valu = [&](auto jc) __attribute__((always_inline)) {
    constexpr int J = decltype(jc)::value;
    if constexpr (J == 0) {
      const bool full = need_mask | !have_ref;  // scalar flags: one branch on the hot path
      if (__builtin_expect(full, 0)) {  // wave-uniform, rare: laid out off the hot path
        if (need_mask) {
          // Masked tiles are the few on the diagonal: their kv_pos reads are simply waited
          // for (which also completes every older LDS read, so the counted waits hold).
          u32x4_t kp0 = lds_read_b128<POFF + 0>(paddr), kp1 = lds_read_b128<POFF + 32>(paddr);
          u32x4_t kp2 = lds_read_b128<POFF + 64>(paddr), kp3 = lds_read_b128<POFF + 96>(paddr);
          lgkm_wait<0>(kp0, kp1, kp2, kp3);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int32_t k0 = (int32_t)kp0[r], k1 = (int32_t)kp1[r];
            const int32_t k2 = (int32_t)kp2[r], k3 = (int32_t)kp3[r];
            if (k0 > qp || (BAND && k0 < ql)) s[0 + r] = -INFINITY;
            if (k1 > qp || (BAND && k1 < ql)) s[4 + r] = -INFINITY;
            if (k2 > qp || (BAND && k2 < ql)) s[8 + r] = -INFINITY;
            if (k3 > qp || (BAND && k3 < ql)) s[12 + r] = -INFINITY;
          }
        }
        const float m_step = block_max() * scale_log2;
        raise = m_step > R.m_run + kRescaleSlack;  // true on the first visible block
        const float m_new = raise ? m_step : R.m_run;
        alpha = __builtin_amdgcn_exp2f(R.m_run - (m_new == -INFINITY ? 0.f : m_new));
        R.l_run *= alpha;
        R.m_run = m_new;
        m_use = m_new == -INFINITY ? 0.f : m_new;
        have_ref = __builtin_amdgcn_ballot_w64(m_new == -INFINITY) == 0;
      } else {
        m_use = R.m_run;
      }
      pin(m_use);
    } else {
      if constexpr (J <= 14) {
#pragma unroll
        for (int v = kBound[J - 1]; v < kBound[J]; ++v) {
          e[v] = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, -m_use));
          pin(e[v]);
        }
      }
      if constexpr (J >= 2) {
#pragma unroll
        for (int v = kBound[J - 2]; v < kBound[J - 1]; ++v) finish(v);
      }
    }
  };

  // ---- first half: P(i-1) on the matrix pipe, K fragments of block i+1 requested ----
  auto first = [&](auto mc) __attribute__((always_inline)) {
    constexpr int M = decltype(mc)::value;
    // LDS operations issued after V fragment M: 7 - M later V fragments (two reads each)
    // and M K fragments
    lgkm_wait<14 - 2 * M + M>(R.vf[M]);
    R.o[M & 3] = mfma32(__builtin_bit_cast(bf16x8_t, R.vf[M]),
                        __builtin_bit_cast(bf16x8_t, R.pb[NXT][M >> 2]), R.o[M & 3]);
    R.kf[M] = lds_read_b128<KOFF>(kaddr[M]);
    hook(IntC<M>{});
    valu(IntC<M>{});
    __builtin_amdgcn_sched_barrier(0);
  };
  first(IntC<0>{}); first(IntC<1>{}); first(IntC<2>{}); first(IntC<3>{});
  first(IntC<4>{}); first(IntC<5>{}); first(IntC<6>{}); first(IntC<7>{});

  // ---- second half: Q(i+1) on the matrix pipe, V fragments of block i requested ----
  auto second = [&](auto mc) __attribute__((always_inline)) {
    constexpr int M = decltype(mc)::value;
    // after K fragment M: 7 - M later K fragments and 2 M reads of V fragments
    lgkm_wait<7 - M + 2 * M>(R.kf[M]);
    if constexpr (M == 0) {
      floatx16_t z;
#pragma unroll
      for (int i = 0; i < 16; ++i) z[i] = 0.f;
      R.s[NXT] = mfma32(__builtin_bit_cast(bf16x8_t, R.kf[M]), qf[M], z);
    } else {
      R.s[NXT] = mfma32(__builtin_bit_cast(bf16x8_t, R.kf[M]), qf[M], R.s[NXT]);
    }
    R.vf[M] = lds_read_vt_frag<VOFF + (M >> 2) * 16 * ROW_BYTES>(vaddr[M & 3]);
    hook(IntC<8 + M>{});
    valu(IntC<8 + M>{});
    __builtin_amdgcn_sched_barrier(0);
  };
  second(IntC<0>{}); second(IntC<1>{}); second(IntC<2>{}); second(IntC<3>{});
  second(IntC<4>{}); second(IntC<5>{}); second(IntC<6>{}); second(IntC<7>{});

  // A block of the fast form whose exponentials ran away from the reference (rare): redo
  // its softmax in the full form. No row's sum can pass the test with an infinity or a NaN.
  float blk = lsum0 + lsum1;
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(blk <= kOverflowSum)) != 0, 0)) {
    const float m_step = block_max() * scale_log2;
    const float m_new = fmaxf(R.m_run, m_step);
    m_use = m_new == -INFINITY ? 0.f : m_new;
    const float a2 = __builtin_amdgcn_exp2f(R.m_run - m_use);
    R.l_run *= a2;
    alpha *= a2;
    R.m_run = m_new;
    raise = true;
    lsum0 = lsum1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      e[v] = __builtin_amdgcn_exp2f(fmaf(s[v], scale_log2, -m_use));
      finish(v);
    }
    blk = lsum0 + lsum1;
  }
  R.l_run += blk;
  // rows whose reference maximum moved: bring O to the new reference (rare)
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(raise) != 0, 0)) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) R.o[db][i] *= alpha;
  }
  __builtin_amdgcn_sched_barrier(0);
}

// BAND: packed batch. Positions are shifted per sequence and a query also has a lower bound
// q_lo (the shift of its sequence): visible iff q_lo <= kv_pos <= q_pos.
// SPLIT: the launch splits the KV axis over grid.z and writes fp32 partials to the workspace.
// ACC: the result is merged into a running (O, LSE) in the epilogue instead of being written
// as a partial (Equation 4 applied step by step); see the epilogue.
// ---- ring walk (RING variant): per-shard pointers and the bounded wait for a shard ----
__device__ __forceinline__ int ring_shards(const RingTable& ring) { return ring.n_shards; }
__device__ __forceinline__ int ring_shards(const NoRing&) { return 1; }

// Points the loader at the shard of ring step `shard`. With arrival flags, thread 0 makes
// sure of the step's flag first: `peek` is what it read of that flag while the previous shard
// was being walked (so a shard that arrived in time costs no round trip here); if that was
// zero it polls (uncached loads, a short sleep between them, at most ring.spin_limit of them).
// The whole workgroup learns the outcome through LDS; false = the flag never came up:
// bit `shard` of *ring.error is set and the caller leaves the shard out. Every wait ends.
__device__ __forceinline__ int ring_flag(const RingTable& ring, int step) {
  return __hip_atomic_load(ring.arrived + step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ bool ring_enter(const RingTable& ring, int shard, int kvh, int tid,
                                           int* wg_scratch, int& peek, const char*& k_head,
                                           const char*& v_head, const int32_t*& kv_pos_cur,
                                           const int2*& bounds_cur, int32_t& total_kv,
                                           int& t_end) {
  const RingShard& e = ring.shard[shard];
  total_kv = e.total_kv;
  t_end = e.n_tiles;
  k_head = (const char*)e.k + (int64_t)kvh * ROW_BYTES;
  v_head = (const char*)e.v + (int64_t)kvh * ROW_BYTES;
  kv_pos_cur = e.kv_pos;
  bounds_cur = e.bounds;
  if (ring.arrived == nullptr) return true;
  int* const slot = wg_scratch + 20 + (shard & 1);  // two slots: a wavefront may lag one step
  if (tid == 0) {
    int ok = 1;
    if (peek == 0) {
      int budget = ring.spin_limit;
      while (ring_flag(ring, shard) == 0) {
        if (--budget <= 0) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(32);
      }
    }
    if (!ok) atomicOr(ring.error, 1 << shard);  // which step gave up (n_shards <= 32)
    *slot = ok;
    // a look at the next step's flag, used when the walk gets there
    peek = shard + 1 < ring.n_shards ? ring_flag(ring, shard + 1) : 0;
  }
  lds_barrier();
  const int ok = __builtin_amdgcn_readfirstlane(*slot);
  // The shard's data is read after its flag: every load of it is issued after this barrier,
  // which thread 0 reaches only with the flag's value in hand. No cache invalidation: the
  // caller gives every step a buffer of its own that is complete before its flag is set and
  // is not written again while the kernel runs, so no line of it can be in a cache before the
  // flag is seen. (An agent-scope acquire here invalidates the XCD's L2 once per workgroup and
  // shard and costs 3.5 % of the walk.)
  return ok != 0;
}
__device__ __forceinline__ bool ring_enter(const NoRing&, int, int, int, int*, int&, const char*&,
                                           const char*&, const int32_t*&, const int2*&, int32_t&,
                                           int&) {
  return true;
}

// RING: one launch walks the KV shards of all ring steps of a rank, in ring order, with one
// running (O, l, m) in registers: the merge of Equation 4 happens inside the online softmax
// and nothing but the rank's final output is written. `ring` names the shards (any sizes, empty
// ones included) and, optionally, one arrival flag per step that the workgroup waits for
// (bounded) before it touches the shard.
template <typename TO, bool BAND, bool SPLIT, bool ACC, bool RING>
__device__ __forceinline__ void prefill_body(const Params& p,
                                             const int2* __restrict__ tile_bounds,
                                             const RingArg<RING>& ring) {
  static_assert(!RING || (!BAND && !SPLIT && !ACC), "the ring walk is its own variant");
  extern __shared__ __align__(16) char smem[];
  char* const kbuf0 = smem;
  char* const vbuf0 = smem + OFF_V8;
  int32_t* const posbuf0 = (int32_t*)(smem + OFF_POS8);
  int* const wg_scratch = (int*)(smem + OFF_SCRATCH8);
  int4* const live = (int4*)(smem + OFF_LIVE8);
  const uint32_t smem_lds = (uint32_t)(size_t)(CP_LDS_AS char*)smem;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int n = lane & 31, g = lane >> 5;
  const int row_block = gridDim.x - 1 - blockIdx.x;  // late (heavier) rows first
  const int kvh = blockIdx.y;
  const int split = blockIdx.z;

  // ---- this lane's query row ----
  // (rows fit 31 bits: checked by the launcher)
  const int64_t r = (int64_t)row_block * BM + wave * 32 + n;
  const bool row_ok = r < p.rows;
  const int64_t token = row_ok ? (int64_t)((uint32_t)r / (uint32_t)p.group) : 0;
  const int hg = row_ok ? (int)(r - token * p.group) : 0;
  const int64_t row_lin = (token * p.n_kv_heads + kvh) * p.group + hg;  // index into [tokens, N_H]
  const int32_t qp = row_ok ? p.q_pos[token] : CP_POS_PAD_Q;
  const int32_t ql = BAND && row_ok ? p.q_lo[token] : INT32_MIN;
  int32_t total_kv = p.total_kv;  // (the ring walk sets it, and t_end, per shard)
  const float scale_log2 = p.scale_log2;
  // The start-up chain is q_pos -> visible tiles -> first tile; the bounds of the first 512
  // tiles are requested now so that they arrive together with q_pos, and the Q fragments
  // (needed last) are requested after both and waited for only before the first product.
  const int t_begin = split * p.tiles_per_split;
  int t_end = min(p.n_tiles, t_begin + p.tiles_per_split);
  if constexpr (RING) {
    total_kv = ring.shard[0].total_kv;
    t_end = ring.shard[0].n_tiles;
  }
  int2 first_bounds = make_int2(0, 0);
  const int2* bounds_cur = tile_bounds;
  if constexpr (RING) bounds_cur = ring.shard[0].bounds;
  if (t_begin + wave * 64 + lane < t_end) first_bounds = bounds_cur[t_begin + wave * 64 + lane];

  bf16x8_t qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (row_ok) t = *(const uint4*)(p.q + row_lin * D + ks * 16 + g * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, t);
  }

  // ---- query position range of the wavefront and of the workgroup ----
  // rows that can see anything: a padded query (CP_POS_PAD_Q) and the rows past the end of
  // the shard cannot, and stay out of the ranges below
  const bool sees = row_ok && qp >= 0;
  int w_qmin = sees ? qp : INT32_MAX, w_qmax = qp;
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
  lds_barrier();
  int wg_qmax = INT32_MIN, wg_lomin = INT32_MAX;
#pragma unroll
  for (int w = 0; w < NWAVE; ++w) {
    wg_qmax = max(wg_qmax, wg_scratch[w]);
    if (BAND) wg_lomin = min(wg_lomin, wg_scratch[NWAVE + 1 + w]);
  }
  // wave-uniform by construction; say so, so that control flow stays on the scalar unit
  wg_qmax = __builtin_amdgcn_readfirstlane(wg_qmax);
  w_qmin = __builtin_amdgcn_readfirstlane(w_qmin);
  if (BAND) {
    wg_lomin = __builtin_amdgcn_readfirstlane(wg_lomin);
    w_lomax = __builtin_amdgcn_readfirstlane(w_lomax);
  }

  bool have_ref = false;  // every row of the wavefront has a finite reference maximum
  PipeRegs R;
  // Reference max of scaled scores (log2 domain). A row that can see nothing gets a finite
  // reference no score reaches: its exponentials are all zero whichever softmax form its
  // wavefront takes (so one padded row does not keep the other 31 on the masked form), its
  // denominator stays zero, and the epilogue writes O = 0, LSE = -inf for it.
  R.m_run = sees ? -INFINITY : kDeadRowRef;
  R.l_run = 0.f;        // running denominator over this lane's half of the keys
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) R.o[db][i] = 0.f;

  // ---- tile loader: this wavefront brings rows wave*16 .. wave*16+15 of K and of V, four
  // rows (1 KiB) per instruction and tile; lane l covers row l/16 of the four, chunk position
  // l%16. Part I of a tile is one such instruction for K and one for V. `rows_valid` clamps
  // rows past the end of the shard to its last row (they are masked by their position).
  const uint32_t stride_b = (uint32_t)p.n_kv_heads * ROW_BYTES;  // bytes between tokens
  const int l_row = lane >> 4, l_pos = lane & 15;
  const uint32_t v_chunk = (l_pos ^ ((l_row & 3) * 4)) * 16;
  // (wave-uniform; the ring walk re-points them at every shard)
  const char* k_head = (const char*)p.k + (int64_t)kvh * ROW_BYTES;
  const char* v_head = (const char*)p.v + (int64_t)kvh * ROW_BYTES;
  const int32_t* kv_pos_cur = p.kv_pos;
  auto issue_part = [&](auto ic, int key0, int b) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value;
    const int row = wave * 16 + I * 4 + l_row;
    const uint32_t row_c = (uint32_t)min(row, total_kv - 1 - key0);
    const uint32_t roff = __umul24(row_c, stride_b);
    const uint32_t k_chunk = (l_pos ^ ((I * 4 + l_row) & 15)) * 16;  // row & 15 selects the permutation
    const int64_t tile_off = (int64_t)key0 * stride_b;               // uniform
    load_lds16(k_head + tile_off + (roff + k_chunk),
               kbuf0 + b * KD_BYTES + (wave * 16 + I * 4) * ROW_BYTES);
    load_lds16(v_head + tile_off + (roff + v_chunk),
               vbuf0 + b * KD_BYTES + (wave * 16 + I * 4) * ROW_BYTES);
  };
  // kv_pos of the tile goes through a register (the tail needs the pad value)
  auto load_pos = [&](int key0) -> int32_t {
    if (tid >= TILE) return 0;
    const int key = key0 + tid;
    return key < total_kv ? kv_pos_cur[key] : CP_POS_PAD_KV;
  };
  // a tile pays for the mask when one of its keys can be hidden from one of this wavefront's
  // rows (this includes the tiles that only other wavefronts of the workgroup can see)
  auto tile_needs_mask = [&](int tile, int bmin, int bmax) -> bool {
    return bmax > w_qmin || (tile + 1) * TILE > total_kv || (BAND && bmin < w_lomax);
  };

  // ---- fragment addressing (LDS byte addresses, buffer 0) ----
  // K: lane (n, g) reads chunk 2*ks + g of key row n of a block
  uint32_t kaddr[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
    kaddr[ks] = smem_lds + n * ROW_BYTES + ((2 * ks + g) ^ (n & 15)) * 16;
  // V: in its 16-lane group this lane addresses key vj of four and 8 bytes (4 channels) vq
  const int grp = lane >> 4, vj = (lane & 15) >> 2, vq = lane & 3;
  uint32_t vaddr[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
    vaddr[db] = smem_lds + OFF_V8 + ((grp >> 1) * 4 + vj) * ROW_BYTES + (grp & 1) * 32 +
                (vq >> 1) * 16 + (vq & 1) * 8 + (db ^ vj) * 64;
  uint32_t paddr = smem_lds + OFF_POS8 + g * 16;

  const int n_shards = RING ? ring_shards(ring) : 1;
  int flag_peek = 0;
  for (int shard = 0; shard < n_shards; ++shard) {
    if constexpr (RING) {
      if (!ring_enter(ring, shard, kvh, tid, wg_scratch, flag_peek, k_head, v_head, kv_pos_cur,
                      bounds_cur, total_kv, t_end))
        continue;  // the shard never arrived: reported through ring.error, walk goes on
    }
    for (int c0 = t_begin; c0 < t_end; c0 += MAX_LIVE) {
      // Compact the tiles some query of the workgroup can see (smallest key position not
      // beyond the largest query position) into an ascending list in LDS: (tile, min, max).
      lds_barrier();  // previous chunk (list, tile buffers) fully consumed
      {
        const int t = c0 + wave * 64 + lane;
        int2 b = make_int2(0, 0);
        bool lv = false;
        if (t < t_end) {
          b = (c0 == t_begin && shard == 0) ? first_bounds : bounds_cur[t];
          lv = b.x <= wg_qmax && (!BAND || b.y >= wg_lomin);
        }
        const uint64_t mask = __builtin_amdgcn_ballot_w64(lv);
        if (lane == 0) wg_scratch[wave] = __builtin_popcountll(mask);
        lds_barrier();
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
      lds_barrier();
      const int n_live = __builtin_amdgcn_readfirstlane(wg_scratch[NWAVE]);
      if (n_live == 0) continue;

      // ---- prologue: tile 0 into buffer 0, Q stage of block 0 ----
      int32_t next_pos = 0;
      bool need_mask, next_mask = false;
      int next_key0 = 0;
      auto read_entry = [&](int idx, int& key0, bool& mask_it) {
        const int4 e = live[idx < n_live ? idx : n_live - 1];
        const int tile = __builtin_amdgcn_readfirstlane(e.x);
        key0 = tile * TILE;
        mask_it = tile_needs_mask(tile, __builtin_amdgcn_readfirstlane(e.y),
                                  __builtin_amdgcn_readfirstlane(e.z));
      };
      {
        int key0;
        read_entry(0, key0, need_mask);
        read_entry(1, next_key0, next_mask);
        issue_part(IntC<0>{}, key0, 0);
        issue_part(IntC<1>{}, key0, 0);
        issue_part(IntC<2>{}, key0, 0);
        issue_part(IntC<3>{}, key0, 0);
        const int32_t pos = load_pos(key0);
        if (tid < TILE) posbuf0[tid] = pos;
        __syncthreads();  // waits for the tile (vmcnt) and publishes it
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) R.kf[ks] = lds_read_b128<0>(kaddr[ks]);
        lgkm_wait<0>(R.kf[0], R.kf[1], R.kf[2], R.kf[3]);
        lgkm_wait<0>(R.kf[4], R.kf[5], R.kf[6], R.kf[7]);
#pragma unroll
        for (int i = 0; i < 16; ++i) R.s[0][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          R.s[0] = mfma32(__builtin_bit_cast(bf16x8_t, R.kf[ks]), qf[ks], R.s[0]);
        __builtin_amdgcn_sched_barrier(0);
        // stand-in V fragments for the empty P stage of the first step (finite data, P = 0)
#pragma unroll
        for (int m = 0; m < 8; ++m) R.vf[m] = lds_read_vt_frag<0>(vaddr[m & 3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) R.pb[1][0][i] = R.pb[1][1][i] = 0u;
        __builtin_amdgcn_sched_barrier(0);
      }

      auto no_hook = [](auto) {};
      for (int it = 0; it < n_live; ++it) {
        const bool has_next = it + 1 < n_live;
        const int nb = (it + 1) & 1;
        // The next tile is requested during the first two steps, one part (a K and a V
        // instruction per wavefront) at a time: a burst of all eight fills the memory pipeline's
        // queue and stalls every wavefront behind it.
        pipe_body<0, BAND>(R, qf, kaddr, vaddr, paddr, qp, ql, scale_log2, need_mask, have_ref,
                           [&](auto mc) __attribute__((always_inline)) {
                             constexpr int M = decltype(mc)::value;
                             if (M == 1 && __builtin_expect(has_next, 1)) issue_part(IntC<0>{}, next_key0, nb);
                             if (M == 9 && __builtin_expect(has_next, 1)) issue_part(IntC<1>{}, next_key0, nb);
                           });
        pipe_body<1, BAND>(R, qf, kaddr, vaddr, paddr, qp, ql, scale_log2, need_mask, have_ref,
                           [&](auto mc) __attribute__((always_inline)) {
                             constexpr int M = decltype(mc)::value;
                             if (M == 1 && __builtin_expect(has_next, 1)) issue_part(IntC<2>{}, next_key0, nb);
                             if (M == 9 && __builtin_expect(has_next, 1)) {
                               issue_part(IntC<3>{}, next_key0, nb);
                               next_pos = load_pos(next_key0);
                             }
                           });
        pipe_body<2, BAND>(R, qf, kaddr, vaddr, paddr, qp, ql, scale_log2, need_mask, have_ref, no_hook);
        // barrier Y: the next tile has landed in every wavefront
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        if (has_next && tid < TILE) posbuf0[nb * TILE + tid] = next_pos;
        const bool cur_mask = need_mask;
        need_mask = next_mask;
        read_entry(it + 2, next_key0, next_mask);  // no direct-to-LDS load is in flight here
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kaddr[ks] ^= KD_BYTES;  // K of the next tile from here on
        pipe_body<3, BAND>(R, qf, kaddr, vaddr, paddr, qp, ql, scale_log2, cur_mask, have_ref, no_hook);
        // barrier X: every LDS read of this tile has completed; its buffers may be refilled
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        __syncthreads();
#pragma unroll
        for (int db = 0; db < 4; ++db) vaddr[db] ^= KD_BYTES;
        paddr ^= POS_BYTES;
      }

      // ---- drain: P stage of the last block ----
      {
        auto last = [&](auto mc) __attribute__((always_inline)) {
          constexpr int M = decltype(mc)::value;
          lgkm_wait<14 - 2 * M>(R.vf[M]);
          R.o[M & 3] = mfma32(__builtin_bit_cast(bf16x8_t, R.vf[M]),
                              __builtin_bit_cast(bf16x8_t, R.pb[1][M >> 2]), R.o[M & 3]);
        };
        last(IntC<0>{}); last(IntC<1>{}); last(IntC<2>{}); last(IntC<3>{});
        last(IntC<4>{}); last(IntC<5>{}); last(IntC<6>{}); last(IntC<7>{});
        __builtin_amdgcn_sched_barrier(0);
      }
      // back to buffer-0 addressing for the next chunk
      if (n_live & 1) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kaddr[ks] ^= KD_BYTES;
#pragma unroll
        for (int db = 0; db < 4; ++db) vaddr[db] ^= KD_BYTES;
        paddr ^= POS_BYTES;
      }
    }
  }

  // ---- epilogue ----
  static_assert(!(ACC && SPLIT), "the running result is merged by unsplit launches only");
  const float l_tot = R.l_run + xor32(R.l_run);
  float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse_val =
      l_tot > 0.f ? (R.m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  constexpr bool direct = !SPLIT;
  // ACC: weights of Equation 4 for the pair (running result, this step). a_old scales the
  // stored row, the step's row is scaled on its way into the staging buffer. A row the step
  // saw nothing of keeps its stored value (a_old = 1, nothing staged): it is not touched at
  // all unless this is the step that writes the final output.
  float a_old = 0.f;
  if (ACC) {
    const float lse_old = row_ok ? p.lse[row_lin] : -INFINITY;
    const float m = fmaxf(lse_old, lse_val);
    const float w_old = m == -INFINITY ? 0.f : __expf(lse_old - m);
    const float w_cur = m == -INFINITY ? 0.f : __expf(lse_val - m);
    const float den = w_old + w_cur;
    const float rden = den > 0.f ? 1.f / den : 0.f;
    a_old = l_tot > 0.f ? w_old * rden : 1.f;
    inv *= w_cur * rden;
    const float lse_new = den > 0.f ? m + __logf(den) : -INFINITY;
    if (row_ok && g == 0) {
      if (l_tot > 0.f) p.lse[row_lin] = lse_new;
      if (p.final_lse != nullptr) p.final_lse[row_lin] = lse_new;
    }
  } else {
    float* const lse_dst = direct ? p.lse : p.part_lse + (int64_t)split * p.rows_all_heads;
    if (row_ok && g == 0) lse_dst[row_lin] = lse_val;
  }

  // Transpose through LDS (the tile buffers are dead once every wavefront has left the walk;
  // each wavefront then uses a private region). Accumulator (db, i) of lane (n, g) is channel
  // db*32 + (i/4)*8 + g*4 + i%4 of query n.
  __syncthreads();
  char* const stage = smem + wave * 32 * OUT_STRIDE;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int d0 = db * 32 + i4 * 8 + g * 4;
      floatx4_t w = {R.o[db][i4 * 4 + 0] * inv, R.o[db][i4 * 4 + 1] * inv,
                     R.o[db][i4 * 4 + 2] * inv, R.o[db][i4 * 4 + 3] * inv};
      *(floatx4_t*)(stage + n * OUT_STRIDE + d0 * 4) = w;
    }
  wave_lds_fence();
  const int64_t r0 = (int64_t)row_block * BM + wave * 32;
  const bool to_final = !ACC || p.final_out != nullptr;  // uniform
  if (ACC && !to_final) {
    // running result updated in place, 2 rows per pass; rows the step did not see are skipped
    float* const o = p.acc;
    const bool seen = l_tot > 0.f;
#pragma unroll
    for (int pass = 0; pass < 16; ++pass) {
      const int rr = pass * 2 + (lane >> 5), c = (lane & 31) * 4;
      const int64_t rl = __shfl(row_lin, rr, 64);
      const float ao = __shfl(a_old, rr, 64);
      const bool touch = __shfl((int)seen, rr, 64) != 0 && r0 + rr < p.rows;
      floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      if (touch) {
        if (ao != 0.f) {
          const floatx4_t old = *(const floatx4_t*)(o + rl * D + c);
#pragma unroll
          for (int x = 0; x < 4; ++x) a[x] = fmaf(ao, old[x], a[x]);
        }
        *(floatx4_t*)(o + rl * D + c) = a;
      }
    }
  } else if (direct && sizeof(TO) == 2) {
    // 4 rows per pass: 16 lanes x 8 channels each
    bf16_t* const o = (bf16_t*)(ACC ? p.final_out : p.out);
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int rr = pass * 4 + (lane >> 4), c = (lane & 15) * 8;
      const int64_t rl = __shfl(row_lin, rr, 64);
      floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      floatx4_t b = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4 + 16);
      if (ACC) {
        const float ao = __shfl(a_old, rr, 64);
        if (ao != 0.f && r0 + rr < p.rows) {
          const floatx4_t oa = *(const floatx4_t*)(p.acc + rl * D + c);
          const floatx4_t ob = *(const floatx4_t*)(p.acc + rl * D + c + 4);
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            a[x] = fmaf(ao, oa[x], a[x]);
            b[x] = fmaf(ao, ob[x], b[x]);
          }
        }
      }
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
    float* const o = ACC ? (float*)p.final_out
                         : direct ? (float*)p.out
                                  : p.part_out + (int64_t)split * p.rows_all_heads * D;
#pragma unroll
    for (int pass = 0; pass < 16; ++pass) {
      const int rr = pass * 2 + (lane >> 5), c = (lane & 31) * 4;
      const int64_t rl = __shfl(row_lin, rr, 64);
      floatx4_t a = *(const floatx4_t*)(stage + rr * OUT_STRIDE + c * 4);
      if (ACC) {
        const float ao = __shfl(a_old, rr, 64);
        if (ao != 0.f && r0 + rr < p.rows) {
          const floatx4_t old = *(const floatx4_t*)(p.acc + rl * D + c);
#pragma unroll
          for (int x = 0; x < 4; ++x) a[x] = fmaf(ao, old[x], a[x]);
        }
      }
      if (r0 + rr < p.rows) *(floatx4_t*)(o + rl * D + c) = a;
    }
  }
}

template <typename TO, bool BAND, bool SPLIT, bool ACC = false>
__global__ __launch_bounds__(NTHREADS) void prefill_mfma_kernel(
    const Params p, const int2* __restrict__ tile_bounds) {
  prefill_body<TO, BAND, SPLIT, ACC, false>(p, tile_bounds, NoRing{});
}

// All ring steps of a rank in one launch (the RING variant of the body).
template <typename TO>
__global__ __launch_bounds__(NTHREADS) void prefill_ring_walk_kernel(const Params p,
                                                                     const RingTable ring) {
  prefill_body<TO, false, false, false, true>(p, p.bounds, ring);
}
