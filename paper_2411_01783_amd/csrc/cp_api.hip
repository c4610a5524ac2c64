// C-ABI entry points: host-side argument checks, kernel selection, ring drivers.
#include <math.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "cp_common.h"

using namespace cp;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

int check_shape(const cp_shape* s) {
  if (s == nullptr) return CP_ERR_NULL;
  if (s->dtype != CP_BF16 && s->dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if (s->head_dim != 64 && s->head_dim != 128) return CP_ERR_UNSUPPORTED;
  if (s->n_q_heads < 1 || s->n_kv_heads < 1 || s->n_q_heads % s->n_kv_heads != 0)
    return CP_ERR_SHAPE;
  if (s->batch < 1 || s->total_q < 0 || s->total_kv < 0) return CP_ERR_SHAPE;
  if (s->total_q > 0x7fffffffLL || s->total_kv > 0x7fffffffLL) return CP_ERR_SHAPE;
  if ((s->flags & ~CP_SHAPE_UNIQUE_BID) != 0 || s->reserved_f != 0.f) return CP_ERR_SHAPE;
  if (!(s->softmax_scale == s->softmax_scale) || isinf(s->softmax_scale)) return CP_ERR_SHAPE;
  return CP_OK;
}

inline float resolve_scale(float scale, int head_dim) {
  return scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
}

inline bool mfma_prefill_applies(const cp_shape& s) {
  return s.dtype == CP_BF16 && s.head_dim == 128 && (s.n_q_heads / s.n_kv_heads) <= 64;
}

inline size_t elem_size(int32_t dtype) { return dtype == CP_FP32 ? 4 : 2; }

}  // namespace

// Scratch of cp_attn_decode_static: split-KV partials live here instead of in a caller's
// workspace, so that the call allocates nothing. Every GPU holds its own copy of the array at
// its own address; in host code the array's name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[CP_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CP_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return CP_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return CP_OK;
}

}  // namespace

extern "C" {

int cp_version(void) { return 100; }

const char* cp_strerror(int status) {
  switch (status) {
    case CP_OK: return "ok";
    case CP_ERR_NULL: return "a required pointer is NULL";
    case CP_ERR_SHAPE: return "invalid or inconsistent shape";
    case CP_ERR_UNSUPPORTED: return "dtype / head_dim / combination not supported";
    case CP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CP_ERR_LAUNCH: return "HIP kernel launch failed";
    case CP_ERR_ALIGN: return "tensor pointer is not 16-byte aligned";
    default: return "unknown status";
  }
}

int cp_shard_positions(int64_t total, int64_t offset, int32_t n_ranks, int32_t rank,
                       int32_t* pos_out, int64_t* n_out) {
  if (n_out == nullptr) return CP_ERR_NULL;
  if (total < 0 || n_ranks < 1 || rank < 0 || rank >= n_ranks) return CP_ERR_SHAPE;
  if (offset < 0 || total + offset > 0x7fffffffLL) return CP_ERR_SHAPE;
  const int64_t n_chunks = 2 * (int64_t)n_ranks;
  const int64_t size = (total + n_chunks - 1) / n_chunks;
  const int64_t chunk[2] = {rank, n_chunks - 1 - rank};
  int64_t n = 0;
  for (int c = 0; c < 2; ++c) {
    const int64_t lo = std::min(chunk[c] * size, total);
    const int64_t hi = std::min((chunk[c] + 1) * size, total);
    for (int64_t p = lo; p < hi; ++p, ++n)
      if (pos_out != nullptr) pos_out[n] = (int32_t)(p + offset);
  }
  *n_out = n;
  return CP_OK;
}

size_t cp_workspace_bytes(const cp_shape* shape, int32_t kind) {
  if (check_shape(shape) != CP_OK) return 0;
  switch (kind) {
    case CP_WS_PARTIAL:
      if (!mfma_prefill_applies(*shape)) return 0;
      return prefill_mfma_workspace_bytes(*shape) +
             (shape->batch > 1
                  ? varseq_layout(shape->batch, shape->total_q, shape->total_kv).total
                  : 0);
    case CP_WS_DECODE:
      return decode_workspace_bytes(*shape);
    default:
      return 0;
  }
}

int cp_attn_partial(const cp_shape* shape, const void* q, const void* k, const void* v,
                    const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_seqlens_q,
                    const int32_t* cu_seqlens_kv, void* out, float* lse, int32_t out_dtype,
                    void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != CP_OK) return rc;
  const cp_shape& s = *shape;
  if (out_dtype != CP_BF16 && out_dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if ((cu_seqlens_q == nullptr) != (cu_seqlens_kv == nullptr)) return CP_ERR_NULL;
  if (cu_seqlens_q == nullptr && s.batch != 1) return CP_ERR_SHAPE;
  if (s.total_q > 0 && (q == nullptr || q_pos == nullptr || out == nullptr || lse == nullptr))
    return CP_ERR_NULL;
  if (s.total_q > 0 && s.total_kv > 0 && (k == nullptr || v == nullptr || kv_pos == nullptr))
    return CP_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return CP_ERR_ALIGN;
  if (s.total_q == 0) return CP_OK;
  const float scale = resolve_scale(s.softmax_scale, s.head_dim);
  hipStream_t st = (hipStream_t)stream;
  if (mfma_prefill_applies(s) && (cu_seqlens_q == nullptr || s.batch == 1)) {
    const size_t need = prefill_mfma_workspace_bytes(s);
    if (need > 0 && (workspace == nullptr || !aligned256(workspace) || workspace_bytes < need))
      return CP_ERR_WORKSPACE;
    return launch_prefill_mfma(s, scale, q, k, v, q_pos, kv_pos, out, lse, out_dtype, workspace,
                               workspace_bytes, nullptr, nullptr, st);
  }
  if (mfma_prefill_applies(s)) {
    // packed batch: shift every sequence into its own position range, then one launch
    if (s.total_q > 0x7fffffffLL || s.total_kv > 0x7fffffffLL) return CP_ERR_SHAPE;
    const VarseqLayout vl = varseq_layout(s.batch, s.total_q, s.total_kv);
    const size_t need = vl.total + prefill_mfma_workspace_bytes(s);
    if (workspace == nullptr || !aligned256(workspace) || workspace_bytes < need)
      return CP_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    if (launch_varseq_encode(s.batch, s.total_q, s.total_kv, q_pos, kv_pos, cu_seqlens_q,
                             cu_seqlens_kv, ws, st) != CP_OK)
      return CP_ERR_LAUNCH;
    return launch_prefill_mfma(s, scale, q, k, v, (const int32_t*)(ws + vl.q_hi_off),
                               (const int32_t*)(ws + vl.kv_off), out, lse, out_dtype,
                               ws + vl.total, workspace_bytes - vl.total, nullptr,
                               (const int32_t*)(ws + vl.q_lo_off), st);
  }
  return launch_partial_generic(s, scale, q, k, v, q_pos, kv_pos, cu_seqlens_q, cu_seqlens_kv,
                                out, lse, out_dtype, st);
}

int cp_attn_partial_accumulate(const cp_shape* shape, const void* q, const void* k,
                               const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                               float* acc_out, float* acc_lse, void* final_out,
                               int32_t final_dtype, float* final_lse, void* workspace,
                               size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != CP_OK) return rc;
  const cp_shape& s = *shape;
  if (final_out != nullptr && final_dtype != CP_BF16 && final_dtype != CP_FP32)
    return CP_ERR_UNSUPPORTED;
  if (s.batch != 1 || !mfma_prefill_applies(s) || prefill_mfma_splits_kv(s, true))
    return CP_ERR_UNSUPPORTED;
  if (s.total_q > 0 && (q == nullptr || q_pos == nullptr || acc_out == nullptr || acc_lse == nullptr))
    return CP_ERR_NULL;
  if (s.total_q > 0 && s.total_kv > 0 && (k == nullptr || v == nullptr || kv_pos == nullptr))
    return CP_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(acc_out) || !aligned16(final_out))
    return CP_ERR_ALIGN;
  if (s.total_q == 0) return CP_OK;
  const size_t need = prefill_mfma_workspace_bytes(s);
  if (need > 0 && (workspace == nullptr || !aligned256(workspace) || workspace_bytes < need))
    return CP_ERR_WORKSPACE;
  const PrefillAccumulate acc = {acc_out, acc_lse, final_out, final_lse, final_dtype};
  return launch_prefill_mfma(s, resolve_scale(s.softmax_scale, s.head_dim), q, k, v, q_pos, kv_pos,
                             nullptr, nullptr, CP_FP32, workspace, workspace_bytes, nullptr,
                             nullptr, (hipStream_t)stream, &acc);
}

// Argument checks shared by cp_attn_decode and cp_attn_decode_static. Returns CP_OK with
// *launch = false when there is nothing to do.
static int check_decode(const cp_shape* shape, const void* q, const void* k, const void* v,
                        const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_seqlens_kv,
                        const int32_t* bid, const void* out, const float* lse, int32_t out_dtype,
                        bool* launch) {
  *launch = false;
  int rc = check_shape(shape);
  if (rc != CP_OK) return rc;
  const cp_shape& s = *shape;
  if (out_dtype != CP_BF16 && out_dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if (s.dtype != CP_BF16 || s.head_dim != 128) return CP_ERR_UNSUPPORTED;
  if (s.n_q_heads / s.n_kv_heads > 16) return CP_ERR_UNSUPPORTED;
  if (cu_seqlens_kv == nullptr) return CP_ERR_NULL;
  if (s.total_q > 0 &&
      (q == nullptr || q_pos == nullptr || bid == nullptr || out == nullptr || lse == nullptr))
    return CP_ERR_NULL;
  if (s.total_q > 0 && s.total_kv > 0 && (k == nullptr || v == nullptr || kv_pos == nullptr))
    return CP_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return CP_ERR_ALIGN;
  *launch = s.total_q > 0;
  return CP_OK;
}

int cp_attn_decode(const cp_shape* shape, const void* q, const void* k, const void* v,
                   const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_seqlens_kv,
                   const int32_t* bid, void* out, float* lse, int32_t out_dtype,
                   void* workspace, size_t workspace_bytes, void* stream) {
  bool launch = false;
  const int rc = check_decode(shape, q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid, out, lse,
                              out_dtype, &launch);
  if (rc != CP_OK || !launch) return rc;
  const cp_shape& s = *shape;
  const size_t need = decode_workspace_bytes(s);
  if (need > 0 && (workspace == nullptr || !aligned256(workspace) || workspace_bytes < need))
    return CP_ERR_WORKSPACE;
  const float scale = resolve_scale(s.softmax_scale, s.head_dim);
  return launch_decode(s, scale, q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid, out, lse, out_dtype,
                       workspace, workspace_bytes, (hipStream_t)stream);
}

int cp_attn_decode_static(const cp_shape* shape, const void* q, const void* k, const void* v,
                          const int32_t* q_pos, const int32_t* kv_pos,
                          const int32_t* cu_seqlens_kv, const int32_t* bid, void* out, float* lse,
                          int32_t out_dtype, void* stream) {
  bool launch = false;
  const int rc = check_decode(shape, q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid, out, lse,
                              out_dtype, &launch);
  if (rc != CP_OK || !launch) return rc;
  const cp_shape& s = *shape;
  if (decode_workspace_bytes(s) > CP_STATIC_SCRATCH_BYTES) return CP_ERR_WORKSPACE;
  void* ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs != CP_OK) return rs;
  const float scale = resolve_scale(s.softmax_scale, s.head_dim);
  return launch_decode(s, scale, q, k, v, q_pos, kv_pos, cu_seqlens_kv, bid, out, lse, out_dtype,
                       ws, CP_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
}

int cp_attn_merge(int64_t rows, int32_t head_dim, int32_t n_parts, const void* const* outs,
                  const float* const* lses, int32_t part_dtype, void* out, int32_t out_dtype,
                  float* lse_out, void* stream) {
  if (rows < 0 || head_dim < 8 || head_dim > 256 || head_dim % 8 != 0) return CP_ERR_SHAPE;
  if (n_parts < 1 || n_parts > CP_MAX_PARTS) return CP_ERR_SHAPE;
  if ((part_dtype != CP_BF16 && part_dtype != CP_FP32) ||
      (out_dtype != CP_BF16 && out_dtype != CP_FP32))
    return CP_ERR_UNSUPPORTED;
  if (outs == nullptr || lses == nullptr) return CP_ERR_NULL;
  if (rows > 0) {
    if (out == nullptr) return CP_ERR_NULL;
    for (int s = 0; s < n_parts; ++s) {
      if (outs[s] == nullptr || lses[s] == nullptr) return CP_ERR_NULL;
      if (!aligned16(outs[s])) return CP_ERR_ALIGN;
    }
    if (!aligned16(out)) return CP_ERR_ALIGN;
  }
  if (rows == 0) return CP_OK;
  return launch_merge(rows, head_dim, n_parts, outs, lses, part_dtype, out, out_dtype, lse_out,
                      (hipStream_t)stream);
}

}  // extern "C"

// ---------------------------------------------------------------------------
// ring drivers
// ---------------------------------------------------------------------------

// Prefill drivers over packed batches (the fused variable-length inputs of Algorithm 2): every
// rank's Q and KV hold `batch` sequences back to back with per-rank cu_seqlens.
static bool ring_is_packed(const cp_ring_desc* d, bool decode) {
  return !decode && d->cu_seqlens_q != nullptr;
}

static int check_ring(const cp_ring_desc* d, bool decode) {
  if (d == nullptr) return CP_ERR_NULL;
  if (d->n_ranks < 1 || d->n_ranks > CP_MAX_PARTS) return CP_ERR_SHAPE;
  if (d->fused_merge < 0 || d->fused_merge > 2) return CP_ERR_SHAPE;
  if (d->message_layout != 0 && d->message_layout != 1) return CP_ERR_SHAPE;
  if (d->gathered_q != 0 && d->gathered_q != 1) return CP_ERR_SHAPE;
  if (d->unique_bid != 0 && d->unique_bid != 1) return CP_ERR_SHAPE;
  if (d->gathered_q && (!d->keep_partials || d->message_layout || d->fused_merge))
    return CP_ERR_UNSUPPORTED;
  if (d->fused_merge && (decode || d->keep_partials || d->part_dtype != CP_FP32))
    return CP_ERR_UNSUPPORTED;
  if (d->n_q == nullptr || d->n_kv == nullptr || d->q == nullptr || d->k == nullptr ||
      d->v == nullptr || d->q_pos == nullptr || d->kv_pos == nullptr || d->out == nullptr)
    return CP_ERR_NULL;
  if (d->fused_merge == 2 && d->arrived != nullptr &&
      (d->ring_error == nullptr || d->spin_limit < 1))
    return CP_ERR_SHAPE;
  if (d->partial_out == nullptr || (d->partial_lse == nullptr && !d->message_layout))
    return CP_ERR_NULL;
  if (d->part_dtype != CP_BF16 && d->part_dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if (d->out_dtype != CP_BF16 && d->out_dtype != CP_FP32) return CP_ERR_UNSUPPORTED;
  if (!aligned16(d->partial_out)) return CP_ERR_ALIGN;
  if (decode) {
    if (d->batch < 1 || d->cu_seqlens_kv == nullptr || d->bid == nullptr) return CP_ERR_NULL;
  }
  const bool packed = ring_is_packed(d, decode);
  if (packed) {
    if (d->batch < 1) return CP_ERR_SHAPE;
    if (d->cu_seqlens_kv == nullptr) return CP_ERR_NULL;
    if (d->fused_merge || d->gathered_q || d->aux_stream != nullptr) return CP_ERR_UNSUPPORTED;
  }
  cp_shape s = {};
  s.dtype = d->dtype; s.head_dim = d->head_dim; s.n_q_heads = d->n_q_heads;
  s.n_kv_heads = d->n_kv_heads; s.batch = (decode || packed) ? d->batch : 1;
  s.softmax_scale = d->softmax_scale;
  int rc = check_shape(&s);
  if (rc != CP_OK) return rc;
  for (int r = 0; r < d->n_ranks; ++r) {
    if (d->n_q[r] < 0 || d->n_kv[r] < 0) return CP_ERR_SHAPE;
    if (d->n_q[r] > 0 && (d->q[r] == nullptr || d->q_pos[r] == nullptr || d->out[r] == nullptr))
      return CP_ERR_NULL;
    if (d->n_kv[r] > 0 && (d->k[r] == nullptr || d->v[r] == nullptr || d->kv_pos[r] == nullptr))
      return CP_ERR_NULL;
    if (decode && (d->cu_seqlens_kv[r] == nullptr || (d->n_q[r] > 0 && d->bid[r] == nullptr)))
      return CP_ERR_NULL;
    if (packed && (d->cu_seqlens_q[r] == nullptr || d->cu_seqlens_kv[r] == nullptr))
      return CP_ERR_NULL;
  }
  return CP_OK;
}

static cp_shape ring_shape(const cp_ring_desc* d, int q_rank, int kv_rank, bool decode) {
  cp_shape s = {};
  s.dtype = d->dtype; s.head_dim = d->head_dim; s.n_q_heads = d->n_q_heads;
  s.n_kv_heads = d->n_kv_heads; s.batch = (decode || ring_is_packed(d, decode)) ? d->batch : 1;
  s.total_q = d->n_q[q_rank]; s.total_kv = d->n_kv[kv_rank];
  s.softmax_scale = d->softmax_scale;
  if (decode && d->unique_bid) s.flags = CP_SHAPE_UNIQUE_BID;
  return s;
}

// Ring workspace layout: the per-tile kv_pos bounds of every rank's KV shard (computed once
// per driver call, reused by the N calls that read the shard), then the per-call workspace.
static bool ring_uses_tile_bounds(const cp_ring_desc* d, bool decode) {
  cp_shape s = ring_shape(d, 0, 0, decode);
  // (a packed batch shifts its positions per call, so bounds of the raw positions are no use)
  return !decode && !ring_is_packed(d, decode) && mfma_prefill_applies(s);
}

static size_t ring_bounds_bytes(const cp_ring_desc* d, bool decode) {
  if (!ring_uses_tile_bounds(d, decode)) return 0;
  size_t total = 0;
  for (int b = 0; b < d->n_ranks; ++b) total += kv_tile_bounds_bytes(d->n_kv[b]);
  return total;
}

// Shape of the one decode call KV holder b answers with when the queries are gathered.
static cp_shape gathered_decode_shape(const cp_ring_desc* d, int b) {
  cp_shape s = ring_shape(d, 0, b, true);
  s.total_q = 0;
  for (int a = 0; a < d->n_ranks; ++a) s.total_q += d->n_q[a];
  return s;
}

extern "C" size_t cp_ring_workspace_bytes(const cp_ring_desc* d, int32_t decode) {
  if (check_ring(d, decode != 0) != CP_OK) return 0;
  size_t need = 0;
  for (int a = 0; a < d->n_ranks; ++a)
    for (int b = 0; b < d->n_ranks; ++b) {
      cp_shape s = ring_shape(d, a, b, decode != 0);
      need = std::max(need, cp_workspace_bytes(&s, decode ? CP_WS_DECODE : CP_WS_PARTIAL));
    }
  if (d->gathered_q) {
    for (int b = 0; b < d->n_ranks; ++b) {
      cp_shape s = ring_shape(d, 0, b, decode != 0);
      s.total_q = 0;
      for (int a = 0; a < d->n_ranks; ++a) s.total_q += d->n_q[a];
      need = std::max(need, cp_workspace_bytes(&s, decode ? CP_WS_DECODE : CP_WS_PARTIAL));
    }
    if (decode) {
      size_t regions = 0;
      bool flat = true;
      for (int b = 0; b < d->n_ranks; ++b) {
        const cp_shape s = gathered_decode_shape(d, b);
        flat = flat && decode_flat_applies(s);
        regions += decode_flat_region_bytes(s);
      }
      if (flat) need = std::max(need, regions);
    }
  }
  return need + ring_bounds_bytes(d, decode != 0);
}

namespace {

// Where the partial (O, LSE) of a slot live. Two buffers, or (message_layout) one buffer of
// messages, each the slot's O followed by its LSE: what the All2All of Algorithms 3 and 4
// moves as one piece, written in place by the attention kernel and read in place by the merge.
struct RingSlots {
  int64_t max_q = 0;
  size_t out_slot_bytes = 0;
  size_t lse_slot_elems = 0;
  size_t out_stride = 0;   // bytes between the O of consecutive slots
  bool messages = false;
  char* out_base = nullptr;
  float* lse_base = nullptr;
  void* out(int64_t slot) const { return out_base + slot * out_stride; }
  float* lse(int64_t slot) const {
    return messages ? (float*)(out_base + slot * out_stride + out_slot_bytes)
                    : lse_base + slot * lse_slot_elems;
  }
};

size_t ring_message_bytes(size_t out_slot_bytes, size_t lse_slot_elems) {
  return (out_slot_bytes + lse_slot_elems * sizeof(float) + 255) / 256 * 256;
}

RingSlots make_slots(const cp_ring_desc* d) {
  RingSlots r;
  for (int i = 0; i < d->n_ranks; ++i) r.max_q = std::max<int64_t>(r.max_q, d->n_q[i]);
  r.lse_slot_elems = (size_t)r.max_q * d->n_q_heads;
  r.out_slot_bytes = r.lse_slot_elems * d->head_dim * elem_size(d->part_dtype);
  r.messages = d->message_layout != 0;
  r.out_stride = r.messages ? ring_message_bytes(r.out_slot_bytes, r.lse_slot_elems)
                            : r.out_slot_bytes;
  r.out_base = (char*)d->partial_out;
  r.lse_base = d->partial_lse;
  return r;
}

struct RingWork {
  bool use_bounds = false;
  bool dual = false;          // alternate the calls of a rank between two streams
  hipStream_t aux = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  size_t bounds_off[CP_MAX_PARTS] = {};
  char* call_ws = nullptr;
  size_t call_ws_bytes = 0;
};

// Checks the workspace and, for the MFMA path, records the tile bounds of every KV shard.
int ring_prepare(const cp_ring_desc* d, bool decode, hipStream_t st, RingWork& w) {
  const size_t need = cp_ring_workspace_bytes(d, decode ? 1 : 0);
  if (need > 0 && (d->workspace == nullptr || !aligned256(d->workspace) ||
                   d->workspace_bytes < need))
    return CP_ERR_WORKSPACE;
  w.use_bounds = ring_uses_tile_bounds(d, decode);
  size_t off = 0;
  if (w.use_bounds) {
    void* bounds[CP_MAX_PARTS];
    for (int b = 0; b < d->n_ranks; ++b) {
      w.bounds_off[b] = off;
      bounds[b] = (char*)d->workspace + off;
      off += kv_tile_bounds_bytes(d->n_kv[b]);
    }
    const int rc = launch_kv_tile_bounds_ring(d->n_ranks, d->kv_pos, d->n_kv, bounds, st);
    if (rc != CP_OK) return rc;
  }
  w.call_ws = (char*)d->workspace + off;
  w.call_ws_bytes = d->workspace_bytes >= off ? d->workspace_bytes - off : 0;
  // Two streams, and the merge fused into the epilogues, only when no call splits its KV axis
  // through the shared per-call scratch.
  bool scratch = !w.use_bounds;
  if (!decode && w.use_bounds && (d->aux_stream != nullptr || d->fused_merge)) {
    for (int a = 0; a < d->n_ranks && !scratch; ++a)
      for (int b = 0; b < d->n_ranks && !scratch; ++b)
        scratch = d->n_q[a] > 0 &&
                  prefill_mfma_splits_kv(ring_shape(d, a, b, false), d->fused_merge != 0);
  }
  if (d->fused_merge && d->n_ranks > 1 && scratch) return CP_ERR_UNSUPPORTED;
  if (d->aux_stream != nullptr && !decode && w.use_bounds && !d->fused_merge) {
    if (!scratch) {
      if (hipEventCreateWithFlags(&w.fork, hipEventDisableTiming) != hipSuccess) return CP_ERR_LAUNCH;
      if (hipEventCreateWithFlags(&w.join, hipEventDisableTiming) != hipSuccess) {
        (void)hipEventDestroy(w.fork);
        return CP_ERR_LAUNCH;
      }
      w.dual = true;
      w.aux = (hipStream_t)d->aux_stream;
    }
  }
  return CP_OK;
}

// Fused merge: the N steps of one rank keep a running (O, LSE) in partial slot 0. Step 0
// writes it, steps 1 .. N-2 merge into it in their epilogues, the last step writes the merged
// O to the rank's output. `kv_of_step(j)` names the KV rank of step j.
template <typename KvOf>
int ring_rank_fused(const cp_ring_desc* d, const RingWork& w, const RingSlots& slots, int a,
                    int n, hipStream_t st, KvOf kv_of_step) {
  float* const acc_o = (float*)slots.out(0);
  float* const acc_l = slots.lse(0);
  float* const lse_out = d->lse != nullptr ? d->lse[a] : nullptr;
  if (d->n_q[a] == 0) return CP_OK;
  int rc = ring_partial(d, w, false, a, kv_of_step(0), acc_o, acc_l, st);
  for (int j = 1; j < n && rc == CP_OK; ++j) {
    const bool last = j == n - 1;
    const PrefillAccumulate acc = {acc_o, acc_l, last ? d->out[a] : nullptr,
                                   last ? lse_out : nullptr, d->out_dtype};
    rc = ring_partial(d, w, false, a, kv_of_step(j), nullptr, nullptr, st, &acc);
  }
  return rc;
}

// fused_merge == 2: all ring steps of rank a in one launch (see launch_prefill_mfma_ring).
// `kv_of_step(j)` names the KV rank of step j.
template <typename KvOf>
int ring_rank_walk(const cp_ring_desc* d, const RingWork& w, const RingSlots& slots, int a,
                   int n, hipStream_t st, KvOf kv_of_step) {
  if (d->n_q[a] == 0) return CP_OK;
  if (!w.use_bounds) return CP_ERR_UNSUPPORTED;
  const void* k[CP_MAX_PARTS];
  const void* v[CP_MAX_PARTS];
  const int32_t* pos[CP_MAX_PARTS];
  const void* bounds[CP_MAX_PARTS];
  int64_t n_kv[CP_MAX_PARTS];
  int64_t largest = 0;
  for (int j = 0; j < n; ++j) {
    const int s = kv_of_step(j);
    if (!aligned16(d->k[s]) || !aligned16(d->v[s])) return CP_ERR_ALIGN;
    k[j] = d->k[s]; v[j] = d->v[s]; pos[j] = d->kv_pos[s]; n_kv[j] = d->n_kv[s];
    bounds[j] = (const char*)d->workspace + w.bounds_off[s];
    largest = std::max(largest, d->n_kv[s]);
  }
  if (!aligned16(d->q[a])) return CP_ERR_ALIGN;
  cp_shape s = ring_shape(d, a, 0, false);
  s.total_kv = largest;
  if (!prefill_ring_walk_applies(s, n)) return CP_ERR_UNSUPPORTED;
  const int32_t* arrived = d->arrived != nullptr ? d->arrived[a] : nullptr;
  float* const lse_out = d->lse != nullptr ? d->lse[a] : nullptr;
  return launch_prefill_mfma_ring(s, resolve_scale(s.softmax_scale, s.head_dim), d->q[a],
                                  d->q_pos[a], n, k, v, pos, bounds, n_kv, arrived,
                                  d->ring_error != nullptr ? d->ring_error + a : nullptr,
                                  d->spin_limit, d->out[a],
                                  lse_out != nullptr ? lse_out : slots.lse(0),  // LSE not wanted
                                  d->out_dtype, st);
}

void ring_finish(RingWork& w) {
  if (w.dual) {
    (void)hipEventDestroy(w.fork);
    (void)hipEventDestroy(w.join);
    w.dual = false;
  }
}

// The N partial calls of one rank: `call(j, stream)` issues step j. With two streams the
// aux stream first waits for everything enqueued on `st` so far (the previous rank's merge
// still reads the slots), and `st` waits for the aux stream before the caller merges.
template <typename Call>
int ring_rank_steps(const RingWork& w, int n, hipStream_t st, Call call) {
  if (w.dual) {
    if (hipEventRecord(w.fork, st) != hipSuccess ||
        hipStreamWaitEvent(w.aux, w.fork, 0) != hipSuccess)
      return CP_ERR_LAUNCH;
  }
  for (int j = 0; j < n; ++j) {
    const int rc = call(j, (w.dual && (j & 1)) ? w.aux : st);
    if (rc != CP_OK) return rc;
  }
  if (w.dual) {
    if (hipEventRecord(w.join, w.aux) != hipSuccess ||
        hipStreamWaitEvent(st, w.join, 0) != hipSuccess)
      return CP_ERR_LAUNCH;
  }
  return CP_OK;
}

// One partial-attention call of the ring: queries of rank `a` against KV of rank `b`.
int ring_partial(const cp_ring_desc* d, const RingWork& w, bool decode, int a, int b, void* o,
                 float* l, hipStream_t st, const PrefillAccumulate* acc = nullptr) {
  cp_shape s = ring_shape(d, a, b, decode);
  if (acc != nullptr && (decode || !w.use_bounds)) return CP_ERR_UNSUPPORTED;
  if (decode)
    return cp_attn_decode(&s, d->q[a], d->k[b], d->v[b], d->q_pos[a], d->kv_pos[b],
                          d->cu_seqlens_kv[b], d->bid[a], o, l, d->part_dtype, w.call_ws,
                          w.call_ws_bytes, st);
  if (w.use_bounds && s.total_q > 0) {
    if (!aligned16(d->q[a]) || !aligned16(d->k[b]) || !aligned16(d->v[b])) return CP_ERR_ALIGN;
    return launch_prefill_mfma(s, resolve_scale(s.softmax_scale, s.head_dim), d->q[a], d->k[b],
                               d->v[b], d->q_pos[a], d->kv_pos[b], o, l, d->part_dtype, w.call_ws,
                               w.call_ws_bytes, (char*)d->workspace + w.bounds_off[b], nullptr, st,
                               acc);
  }
  const bool packed = ring_is_packed(d, decode);
  return cp_attn_partial(&s, d->q[a], d->k[b], d->v[b], d->q_pos[a], d->kv_pos[b],
                         packed ? d->cu_seqlens_q[a] : nullptr,
                         packed ? d->cu_seqlens_kv[b] : nullptr, o, l, d->part_dtype, w.call_ws,
                         w.call_ws_bytes, st);
}

int ring_merge(const cp_ring_desc* d, const RingSlots& slots, int a, int64_t first_slot,
               hipStream_t st) {
  const void* outs[CP_MAX_PARTS];
  const float* lses[CP_MAX_PARTS];
  for (int s = 0; s < d->n_ranks; ++s) {
    outs[s] = slots.out(first_slot + s);
    lses[s] = slots.lse(first_slot + s);
  }
  float* lse_out = d->lse != nullptr ? d->lse[a] : nullptr;
  return cp_attn_merge(d->n_q[a] * d->n_q_heads, d->head_dim, d->n_ranks, outs, lses,
                       d->part_dtype, d->out[a], d->out_dtype, lse_out, st);
}

}  // namespace

extern "C" {

size_t cp_ring_message_bytes(const cp_ring_desc* d) {
  if (d == nullptr || d->n_q == nullptr || d->n_ranks < 1 || d->n_ranks > CP_MAX_PARTS) return 0;
  if (d->part_dtype != CP_BF16 && d->part_dtype != CP_FP32) return 0;
  if (d->n_q_heads < 1 || d->head_dim < 1) return 0;
  for (int i = 0; i < d->n_ranks; ++i)
    if (d->n_q[i] < 0) return 0;
  const RingSlots r = make_slots(d);
  return ring_message_bytes(r.out_slot_bytes, r.lse_slot_elems);
}

int cp_ring_passkv(const cp_ring_desc* d, void* stream) {
  int rc = check_ring(d, false);
  if (rc != CP_OK) return rc;
  if (d->gathered_q) return CP_ERR_UNSUPPORTED;  // pass-Q only
  hipStream_t st = (hipStream_t)stream;
  const RingSlots slots = make_slots(d);
  const int n = d->n_ranks;
  RingWork w;
  rc = ring_prepare(d, false, st, w);
  if (rc != CP_OK) return rc;
  // Algorithm 2 as seen from each rank k in turn: N ring steps, then a local merge.
  for (int k = 0; k < n && rc == CP_OK; ++k) {
    if (d->fused_merge == 2) {
      rc = ring_rank_walk(d, w, slots, k, n, st, [&](int j) { return ((k - j) % n + n) % n; });
      continue;
    }
    if (d->fused_merge && n > 1) {
      rc = ring_rank_fused(d, w, slots, k, n, st, [&](int j) { return ((k - j) % n + n) % n; });
      continue;
    }
    const int64_t base = d->keep_partials ? (int64_t)k * n : 0;
    rc = ring_rank_steps(w, n, st, [&](int j, hipStream_t sj) {
      const int s = ((k - j) % n + n) % n;  // origin rank of the KV held at step j
      return ring_partial(d, w, false, k, s, slots.out(base + s), slots.lse(base + s), sj);
    });
    if (rc == CP_OK) rc = ring_merge(d, slots, k, base, st);
  }
  ring_finish(w);
  return rc;
}

// gathered_q: the query shards of all source ranks lie back to back in one buffer (an
// all-gather of the small Q instead of passing it round), so a KV holder answers all N ring
// steps of Algorithms 3 / 4 with one call over the gathered queries. Its output block, N slots
// of equal size, is the holder's All2All send buffer in destination order.
static bool queries_are_gathered(const cp_ring_desc* d, bool decode) {
  const size_t row = (size_t)d->n_q_heads * d->head_dim * elem_size(d->dtype);
  for (int s = 0; s < d->n_ranks; ++s) {
    if (d->n_q[s] != d->n_q[0] || d->n_q[s] == 0) return false;
    if (s == 0) continue;
    if ((const char*)d->q[s] != (const char*)d->q[s - 1] + d->n_q[s - 1] * row) return false;
    if (d->q_pos[s] != d->q_pos[s - 1] + d->n_q[s - 1]) return false;
    if (decode && d->bid[s] != d->bid[s - 1] + d->n_q[s - 1]) return false;
  }
  return true;
}

static int ring_passq_gathered(const cp_ring_desc* d, bool decode, hipStream_t st) {
  if (!queries_are_gathered(d, decode)) return CP_ERR_UNSUPPORTED;
  const RingSlots slots = make_slots(d);
  const int n = d->n_ranks;
  RingWork w;
  int rc = ring_prepare(d, decode, st, w);
  if (rc != CP_OK) return rc;
  if (decode) {
    // Every holder's split-KV partials into its own region, one merge over splits x holders.
    cp_shape shapes[CP_MAX_PARTS];
    void* regions[CP_MAX_PARTS];
    bool flat = true;
    size_t off = 0;
    for (int k = 0; k < n; ++k) {
      shapes[k] = gathered_decode_shape(d, k);
      flat = flat && decode_flat_applies(shapes[k]);
      regions[k] = w.call_ws + off;
      off += decode_flat_region_bytes(shapes[k]);
    }
    if (flat) {
      if (off > w.call_ws_bytes) return CP_ERR_WORKSPACE;
      for (int k = 0; k < n && rc == CP_OK; ++k) {
        if (!aligned16(d->q[0]) || !aligned16(d->k[k]) || !aligned16(d->v[k])) rc = CP_ERR_ALIGN;
        else
          rc = launch_decode_flat_partials(
              shapes[k], resolve_scale(d->softmax_scale, d->head_dim), d->q[0], d->k[k], d->v[k],
              d->q_pos[0], d->kv_pos[k], d->cu_seqlens_kv[k], d->bid[0], regions[k],
              decode_flat_region_bytes(shapes[k]), st);
      }
      if (rc != CP_OK) return rc;
      const size_t out_row = (size_t)d->n_q_heads * d->head_dim * elem_size(d->out_dtype);
      bool one = true;
      for (int a = 1; a < n && one; ++a) {
        one = (char*)d->out[a] == (char*)d->out[a - 1] + d->n_q[a - 1] * out_row;
        if (d->lse != nullptr)
          one = one && d->lse[a] != nullptr && d->lse[0] != nullptr &&
                d->lse[a] == d->lse[a - 1] + d->n_q[a - 1] * d->n_q_heads;
      }
      if (one)
        return launch_decode_flat_merge(n, shapes, regions, d->cu_seqlens_kv, d->bid[0],
                                        (int64_t)n * d->n_q[0], d->out[0], d->out_dtype,
                                        d->lse != nullptr ? d->lse[0] : nullptr, st);
      for (int a = 0; a < n && rc == CP_OK; ++a)
        rc = launch_decode_flat_merge(n, shapes, regions, d->cu_seqlens_kv, d->bid[a], d->n_q[a],
                                      d->out[a], d->out_dtype,
                                      d->lse != nullptr ? d->lse[a] : nullptr, st);
      return rc;
    }
  }
  for (int k = 0; k < n && rc == CP_OK; ++k) {
    cp_shape s = ring_shape(d, 0, k, decode);
    s.total_q = (int64_t)n * d->n_q[0];
    void* const o = slots.out((int64_t)k * n);
    float* const l = slots.lse((int64_t)k * n);
    if (decode) {
      rc = cp_attn_decode(&s, d->q[0], d->k[k], d->v[k], d->q_pos[0], d->kv_pos[k],
                          d->cu_seqlens_kv[k], d->bid[0], o, l, d->part_dtype, w.call_ws,
                          w.call_ws_bytes, st);
    } else if (w.use_bounds) {
      if (!aligned16(d->q[0]) || !aligned16(d->k[k]) || !aligned16(d->v[k])) rc = CP_ERR_ALIGN;
      else
        rc = launch_prefill_mfma(s, resolve_scale(s.softmax_scale, s.head_dim), d->q[0], d->k[k],
                                 d->v[k], d->q_pos[0], d->kv_pos[k], o, l, d->part_dtype,
                                 w.call_ws, w.call_ws_bytes,
                                 (char*)d->workspace + w.bounds_off[k], nullptr, st, nullptr);
    } else {
      rc = cp_attn_partial(&s, d->q[0], d->k[k], d->v[k], d->q_pos[0], d->kv_pos[k], nullptr,
                           nullptr, o, l, d->part_dtype, w.call_ws, w.call_ws_bytes, st);
    }
  }
  // The All2All: source rank a merges slot k * n + a of every holder k. When the outputs of
  // the ranks lie back to back as the queries do, the N merges are one launch over the
  // holders' whole blocks.
  const size_t out_row = (size_t)d->n_q_heads * d->head_dim * elem_size(d->out_dtype);
  bool one_merge = slots.max_q == d->n_q[0];
  for (int a = 1; a < n && one_merge; ++a) {
    one_merge = (char*)d->out[a] == (char*)d->out[a - 1] + d->n_q[a - 1] * out_row;
    if (d->lse != nullptr)
      one_merge = one_merge && d->lse[a] != nullptr &&
                  d->lse[a] == d->lse[a - 1] + d->n_q[a - 1] * d->n_q_heads;
  }
  if (one_merge && (d->lse == nullptr || d->lse[0] != nullptr) && rc == CP_OK) {
    const void* outs[CP_MAX_PARTS];
    const float* lses[CP_MAX_PARTS];
    for (int k = 0; k < n; ++k) {
      outs[k] = slots.out((int64_t)k * n);
      lses[k] = slots.lse((int64_t)k * n);
    }
    rc = cp_attn_merge((int64_t)n * d->n_q[0] * d->n_q_heads, d->head_dim, n, outs, lses,
                       d->part_dtype, d->out[0], d->out_dtype,
                       d->lse != nullptr ? d->lse[0] : nullptr, st);
    ring_finish(w);
    return rc;
  }
  for (int a = 0; a < n && rc == CP_OK; ++a) {
    const void* outs[CP_MAX_PARTS];
    const float* lses[CP_MAX_PARTS];
    for (int k = 0; k < n; ++k) {
      outs[k] = slots.out((int64_t)k * n + a);
      lses[k] = slots.lse((int64_t)k * n + a);
    }
    float* lse_out = d->lse != nullptr ? d->lse[a] : nullptr;
    rc = cp_attn_merge(d->n_q[a] * d->n_q_heads, d->head_dim, n, outs, lses, d->part_dtype,
                       d->out[a], d->out_dtype, lse_out, st);
  }
  ring_finish(w);
  return rc;
}

static int ring_passq_common(const cp_ring_desc* d, bool decode, void* stream) {
  int rc = check_ring(d, decode);
  if (rc != CP_OK) return rc;
  if (d->fused_merge == 2) return CP_ERR_UNSUPPORTED;  // pass-KV only: the queries stay put
  if (d->gathered_q) return ring_passq_gathered(d, decode, (hipStream_t)stream);
  hipStream_t st = (hipStream_t)stream;
  const RingSlots slots = make_slots(d);
  const int n = d->n_ranks;
  RingWork w;
  rc = ring_prepare(d, decode, st, w);
  if (rc != CP_OK) return rc;
  if (d->keep_partials) {
    // Algorithms 3 / 4 in ring order: at step j rank k holds the queries of rank
    // s = (k - j) mod N. Writing the result to slot [s][k] is the permute + All2All.
    for (int j = 0; j < n && rc == CP_OK; ++j)
      for (int k = 0; k < n && rc == CP_OK; ++k) {
        const int s = ((k - j) % n + n) % n;
        rc = ring_partial(d, w, decode, s, k, slots.out((int64_t)s * n + k),
                          slots.lse((int64_t)s * n + k), st);
      }
    for (int s = 0; s < n && rc == CP_OK; ++s) rc = ring_merge(d, slots, s, (int64_t)s * n, st);
    ring_finish(w);
    return rc;
  }
  // With N reusable slots the same N*N calls are issued grouped by source rank s
  // (for each s the holders k = s, s+1, ... in ring order), so that the N partials of
  // one source are complete, and can be merged, before the slots are reused.
  for (int s = 0; s < n && rc == CP_OK; ++s) {
    if (d->fused_merge && n > 1) {
      rc = ring_rank_fused(d, w, slots, s, n, st, [&](int j) { return (s + j) % n; });
      continue;
    }
    rc = ring_rank_steps(w, n, st, [&](int j, hipStream_t sj) {
      const int k = (s + j) % n;
      return ring_partial(d, w, decode, s, k, slots.out(k), slots.lse(k), sj);
    });
    if (rc == CP_OK) rc = ring_merge(d, slots, s, 0, st);
  }
  ring_finish(w);
  return rc;
}

int cp_ring_passq(const cp_ring_desc* d, void* stream) { return ring_passq_common(d, false, stream); }

int cp_ring_passq_decode(const cp_ring_desc* d, void* stream) {
  return ring_passq_common(d, true, stream);
}

int cp_ring_prefill(const cp_ring_desc* d, const cp_select_params* params, int64_t p_cached,
                    int32_t rule, int32_t* order_out, void* stream) {
  if (d == nullptr || params == nullptr) return CP_ERR_NULL;
  if (d->n_ranks < 1 || d->n_ranks > CP_MAX_PARTS || d->n_q == nullptr) return CP_ERR_SHAPE;
  if (params->n_ranks != d->n_ranks) return CP_ERR_SHAPE;
  int64_t t_new = 0;
  for (int r = 0; r < d->n_ranks; ++r) {
    if (d->n_q[r] < 0) return CP_ERR_SHAPE;
    t_new += d->n_q[r];
  }
  int32_t order = CP_ORDER_PASS_KV;
  const int rc = cp_select_order(params, t_new, p_cached, rule, &order);
  if (rc != CP_OK) return rc;
  if (order_out != nullptr) *order_out = order;
  return order == CP_ORDER_PASS_Q ? cp_ring_passq(d, stream) : cp_ring_passkv(d, stream);
}

}  // extern "C"
