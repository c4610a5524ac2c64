/*
 * cp_attn.h - C ABI of the per-rank hot path of context-parallel ring attention
 * on one MI355X (gfx950).
 *
 * The library computes, for one context-parallel (CP) rank, exact GQA attention
 * of a query shard against one KV shard under a position-based causal mask,
 * returning a partial output and its log-sum-exp, and the LSE-weighted merge of
 * such partials. Drivers iterate N virtual CP ranks on the one GPU in the order
 * of the paper's ring algorithms. No communication is performed.
 *
 * Conventions for every entry point
 *   - Tensors are token-major, as in Section 3.4:
 *       Q   [tokens, n_q_heads,  head_dim]
 *       K,V [tokens, n_kv_heads, head_dim]
 *       O   [tokens, n_q_heads,  head_dim]
 *       LSE [tokens, n_q_heads]            (always fp32, natural log)
 *     densely packed, 16-byte aligned. Query head h reads KV head
 *     h / (n_q_heads / n_kv_heads).
 *   - Pointers marked (device) are HIP device pointers owned by the caller; the
 *     library never allocates, frees or retains device memory and keeps no
 *     state between calls (the one exception, a scratch array inside the
 *     library's device image, is described at cp_attn_decode_static). Pointers
 *     marked (host) are read during the call only.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without synchronising.
 *   - The return value is CP_OK (0) or a negative cp_status. Arguments are
 *     checked on the host before anything is launched; on error nothing is
 *     enqueued. No exception or abort crosses this boundary.
 *   - Outputs are fully overwritten. A query row that sees no key gets O = 0
 *     and LSE = -inf.
 *   - Key j is visible to query i iff kv_pos[j] <= q_pos[i] (and, for packed
 *     batches, both belong to the same sequence). Padding is expressed through
 *     positions: a padded KV slot carries CP_POS_PAD_KV, a padded query row
 *     carries CP_POS_PAD_Q.
 */
#ifndef CP_ATTN_H
#define CP_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CP_POS_PAD_KV INT32_MAX /* never visible to any query */
#define CP_POS_PAD_Q (-1)       /* sees no key */

typedef enum {
  CP_OK = 0,
  CP_ERR_NULL = -1,        /* a required pointer is NULL */
  CP_ERR_SHAPE = -2,       /* negative or inconsistent sizes, head ratio, batch */
  CP_ERR_UNSUPPORTED = -3, /* dtype / head_dim / combination not implemented */
  CP_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned or too small */
  CP_ERR_LAUNCH = -5,      /* HIP reported a launch failure */
  CP_ERR_ALIGN = -6        /* a tensor pointer is not 16-byte aligned */
} cp_status;

typedef enum { CP_BF16 = 0, CP_FP32 = 1 } cp_dtype;

/* Which computation a workspace is sized for (cp_workspace_bytes). */
typedef enum {
  CP_WS_PARTIAL = 0, /* cp_attn_partial  */
  CP_WS_DECODE = 1,  /* cp_attn_decode   */
  CP_WS_MERGE = 2    /* cp_attn_merge (needs none; returns 0) */
} cp_ws_kind;

/*
 * cp_shape.flags. CP_SHAPE_UNIQUE_BID (cp_attn_decode, cp_attn_decode_static): the caller
 * promises that no sequence id occurs twice in `bid`, as in Algorithm 4, where every sequence
 * has exactly one new token. The call may then take a faster path that reads the rank's whole
 * packed KV in equal ranges per workgroup. If the promise is broken, the queries that share a
 * sequence get unspecified results (all accesses stay in bounds). Ignored by other calls.
 */
#define CP_SHAPE_UNIQUE_BID 1

/* Problem shape of one attention call. */
typedef struct {
  int32_t dtype;      /* cp_dtype of Q, K, V */
  int32_t head_dim;   /* 64 or 128 */
  int32_t n_q_heads;  /* N_H  on this GPU */
  int32_t n_kv_heads; /* N_KV on this GPU; divides n_q_heads */
  int32_t batch;      /* number of packed sequences; 1 when cu_seqlens are NULL */
  int32_t flags;      /* 0, or CP_SHAPE_* bits */
  int64_t total_q;    /* packed query tokens  (>= 0) */
  int64_t total_kv;   /* packed KV tokens     (>= 0) */
  float softmax_scale; /* <= 0 selects 1/sqrt(head_dim) (Appendix B) */
  float reserved_f;    /* must be 0 */
} cp_shape;

/*
 * Load-balanced sharding (Section 3.5.1): a sequence of `total` tokens is cut
 * into 2N chunks of ceil(total/2N) tokens (trailing chunks short or empty) and
 * rank i owns chunk i followed by chunk 2N-1-i. Writes the owned positions,
 * each plus `offset`, to pos_out (host, may be NULL to query the count only)
 * and the count to *n_out (host). Host-only; touches no device.
 * The count never exceeds 2*ceil(total/2N).
 */
int cp_shard_positions(int64_t total, int64_t offset, int32_t n_ranks, int32_t rank,
                       int32_t* pos_out, int64_t* n_out);

/*
 * Bytes of device workspace a call of the given kind needs for this shape
 * (an upper bound valid for any positions). 0 if none. Returns 0 for an
 * invalid shape (the call itself will report the error).
 */
size_t cp_workspace_bytes(const cp_shape* shape, int32_t kind);

/*
 * Partial attention of one ring step: O, LSE = Attn(Q, KV) as used in
 * Algorithm 2 ("Compute O_k^s <- GQA(Q_k, KV^s_k)") and Algorithm 3, with O and
 * LSE as defined in Appendix B, over the keys visible under the causal rule of
 * Section 3.5.1.
 *
 *   shape         (host)
 *   q, k, v       (device) dtype shape->dtype
 *   q_pos         (device) int32 [total_q]   absolute positions
 *   kv_pos        (device) int32 [total_kv]
 *   cu_seqlens_q  (device) int32 [batch+1] packed sequence starts, or NULL iff batch == 1
 *   cu_seqlens_kv (device) int32 [batch+1], NULL iff cu_seqlens_q is NULL
 *   out           (device) [total_q, n_q_heads, head_dim] of out_dtype (cp_dtype)
 *   lse           (device) fp32 [total_q, n_q_heads]
 *   workspace     (device) >= cp_workspace_bytes(shape, CP_WS_PARTIAL), 256-byte
 *                 aligned; may be NULL when that size is 0
 *
 * bf16 inputs with head_dim 128 run on the MFMA kernel (fully masked KV tiles
 * are skipped; short query shards are split over the KV axis through the
 * workspace). Other combinations run on an fp32 vector kernel.
 *
 * Packed batches (the fused variable-length inputs of Algorithm 2, Section 3.4):
 * query i of sequence b sees key j iff j belongs to sequence b and
 * kv_pos[j] <= q_pos[i]. On the MFMA kernel the sequences are told apart by
 * shifting sequence b's positions by the sum over earlier sequences of
 * (1 + largest position in it); that sum over the whole batch must stay below
 * 2^31 - 1 (sequences past the limit would see nothing).
 */
int cp_attn_partial(const cp_shape* shape, const void* q, const void* k, const void* v,
                    const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_seqlens_q,
                    const int32_t* cu_seqlens_kv, void* out, float* lse, int32_t out_dtype,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Partial attention merged into a running result: (acc_out, acc_lse) <- merge((acc_out,
 * acc_lse), Attn(Q, KV)) with the merge of Appendix B, Equation 4 (and the LSE of the union
 * of the key sets), which may be applied step by step because it is associative. One launch:
 * the merge happens in the attention kernel's epilogue, so a ring of N steps needs neither N
 * partial buffers nor a merge pass.
 *
 *   acc_out    (device) fp32 [total_q, n_q_heads, head_dim], read and written
 *   acc_lse    (device) fp32 [total_q, n_q_heads], read and written. The first step of a
 *              ring is a plain cp_attn_partial into (acc_out, acc_lse) with out_dtype CP_FP32.
 *   final_out  (device) or NULL. Not NULL (last step): the merged O is written there in
 *              final_dtype and acc_out is left as it was; acc_lse is still updated.
 *   final_lse  (device) fp32 or NULL: a copy of the merged LSE.
 *   other arguments as cp_attn_partial.
 * Rows of which this step sees no key are not touched (with final_out: copied from acc_out).
 * Errors: as cp_attn_partial; CP_ERR_UNSUPPORTED unless the call runs on the MFMA kernel
 * without a KV split (bf16, head_dim 128, batch 1, at least 128 row blocks of 256 rows).
 */
int cp_attn_partial_accumulate(const cp_shape* shape, const void* q, const void* k,
                               const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                               float* acc_out, float* acc_lse, void* final_out,
                               int32_t final_dtype, float* final_lse, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * Decode attention of one pass-Q ring step: Algorithm 4,
 * "O_s^k <- GQA(Q^s_k, KV_k[bid^s_k])". Each of the shape->total_q query tokens
 * (one per travelling sequence) attends to the KV segment of its own sequence
 * inside this rank's packed KV.
 *
 *   shape->batch   number of sequences packed in k, v (size of cu_seqlens_kv - 1)
 *   shape->total_q number of query tokens in this call (may be < batch)
 *   bid    (device) int32 [total_q] sequence id of each query, in [0, batch)
 *   q_pos  (device) int32 [total_q]
 *   kv_pos (device) int32 [total_kv]
 *   cu_seqlens_kv (device) int32 [batch+1]
 *   workspace: cp_workspace_bytes(shape, CP_WS_DECODE) bytes, 256-byte aligned.
 *
 * The KV axis of every sequence is split across workgroups and the split
 * results are combined with the merge rule of Equation 4 before returning
 * (split-KV decode). Requires bf16 and head_dim 128, n_q_heads/n_kv_heads <= 16.
 */
int cp_attn_decode(const cp_shape* shape, const void* q, const void* k, const void* v,
                   const int32_t* q_pos, const int32_t* kv_pos, const int32_t* cu_seqlens_kv,
                   const int32_t* bid, void* out, float* lse, int32_t out_dtype,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * cp_attn_decode for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same
 * computation, arguments, kernels and results as cp_attn_decode, but the split-KV partials go
 * to a scratch array that is part of the library's device image (CP_STATIC_SCRATCH_BYTES per
 * GPU the library runs on, held until the process ends) instead of a caller's workspace. The
 * call allocates and frees nothing; the array's address on the current device is looked up on
 * the first call on that device (hipGetSymbolAddress) and kept.
 *   - CP_ERR_WORKSPACE if cp_workspace_bytes(shape, CP_WS_DECODE) exceeds
 *     CP_STATIC_SCRATCH_BYTES (nothing is launched); CP_ERR_LAUNCH if the address lookup fails;
 *     otherwise the errors of cp_attn_decode.
 *   - Every call on a GPU uses that GPU's one array. Calls on one stream are ordered and safe;
 *     calls that may overlap on one GPU (different streams without an event between them, or
 *     several host threads on different streams) race on it: the caller must order them.
 *   - Nothing in the array has to be cleared between calls: every launch writes each partial
 *     it later reads.
 * This is the library's only state; all other entry points keep none.
 */
#define CP_STATIC_SCRATCH_BYTES (8u << 20)
int cp_attn_decode_static(const cp_shape* shape, const void* q, const void* k, const void* v,
                          const int32_t* q_pos, const int32_t* kv_pos,
                          const int32_t* cu_seqlens_kv, const int32_t* bid, void* out, float* lse,
                          int32_t out_dtype, void* stream);

/*
 * Merge attention, Appendix B Equation 4:
 *   O = sum_s O^s exp(LSE^s - LSE^max) / sum_s exp(LSE^s - LSE^max),
 * and LSE = LSE^max + log sum_s exp(LSE^s - LSE^max). Rows whose partials are
 * all empty (LSE = -inf) give O = 0, LSE = -inf; the O of an empty partial is
 * never read into the result.
 *
 *   rows      number of (token, head) rows = tokens * n_q_heads
 *   head_dim  multiple of 8, <= 256
 *   outs      (host) array of n_parts (device) pointers, each [rows, head_dim] of part_dtype
 *   lses      (host) array of n_parts (device) pointers, each fp32 [rows]
 *   out       (device) [rows, head_dim] of out_dtype
 *   lse_out   (device) fp32 [rows], or NULL
 *   1 <= n_parts <= CP_MAX_PARTS
 */
#define CP_MAX_PARTS 64
int cp_attn_merge(int64_t rows, int32_t head_dim, int32_t n_parts, const void* const* outs,
                  const float* const* lses, int32_t part_dtype, void* out, int32_t out_dtype,
                  float* lse_out, void* stream);

/*
 * Descriptor of a ring over n_ranks virtual CP ranks that all live on this GPU.
 * Per-rank arrays are (host) arrays of length n_ranks.
 */
typedef struct {
  int32_t dtype, head_dim, n_q_heads, n_kv_heads;
  float softmax_scale; /* <= 0 selects 1/sqrt(head_dim) */
  int32_t n_ranks;
  int32_t out_dtype;   /* dtype of the merged outputs */
  int32_t part_dtype;  /* dtype of the partial outputs: CP_FP32 or CP_BF16 */
  const int64_t* n_q;  /* (host) query tokens of rank k */
  const int64_t* n_kv; /* (host) KV tokens of rank k */
  const void* const* q;         /* (host) -> (device) Q_k  [n_q[k], n_q_heads, head_dim] */
  const void* const* k;         /* (host) -> (device) K_k  [n_kv[k], n_kv_heads, head_dim] */
  const void* const* v;         /* (host) -> (device) V_k */
  const int32_t* const* q_pos;  /* (host) -> (device) int32 [n_q[k]] */
  const int32_t* const* kv_pos; /* (host) -> (device) int32 [n_kv[k]] */
  void* const* out;             /* (host) -> (device) merged O_k of out_dtype */
  float* const* lse;            /* (host) -> (device) merged LSE_k, entries or array may be NULL */
  /*
   * Partial-result buffers (device). Slot i holds max_n_q * n_q_heads * head_dim
   * elements of part_dtype in partial_out and max_n_q * n_q_heads floats in
   * partial_lse, where max_n_q = max_k n_q[k]. With keep_partials == 0 there are
   * n_ranks slots, reused for every rank (slot s = KV origin rank in pass-KV,
   * = KV holder rank in pass-Q). With keep_partials != 0 there are
   * n_ranks * n_ranks slots and the partial of queries of rank a against KV of
   * rank b stays in slot a * n_ranks + b.
   */
  void* partial_out;
  float* partial_lse;
  int32_t keep_partials;
  /*
   * 1: prefill drivers merge in the epilogues instead of keeping N partials per rank
   * (cp_attn_partial_accumulate): step 0 of a rank writes a running (O, LSE) into partial
   * slot 0, the following steps merge into it and the last one writes the rank's output.
   * One slot suffices; no merge pass. Requires part_dtype == CP_FP32, keep_partials == 0, no
   * decode, and calls that do not split their KV axis (else CP_ERR_UNSUPPORTED). 0: off.
   * 2 (cp_ring_passkv only): one launch per rank walks the KV shards of all N ring steps in
   * ring order with one running softmax state in registers, so Equation 4 is applied inside
   * the online softmax and only the rank's output is written: no partials, no merge pass, no
   * per-step launch. Same requirements as 1 (decided on the largest KV shard), and
   * n_ranks <= 32. See `arrived` below for how a step waits for its shard.
   */
  int32_t fused_merge;
  void* workspace; /* (device) max over ranks of the per-call workspace */
  size_t workspace_bytes;
  /* decode (cp_ring_passq_decode) and packed prefill batches (cu_seqlens_q below) */
  int32_t batch;                       /* sequences packed in every rank's KV */
  const int32_t* const* cu_seqlens_kv; /* (host) -> (device) int32 [batch+1] per rank */
  const int32_t* const* bid;           /* (host) -> (device) int32 [n_q[k]] per rank */
  /*
   * Optional second HIP stream (default priority), or NULL. When given, the prefill
   * drivers issue the N partial-attention calls of one rank alternately on `stream` and
   * on aux_stream, so that the tail of one call (its last workgroups, its output writes)
   * overlaps the start of the next; both are joined before the rank's merge, and
   * everything the driver enqueues is ordered after prior work on `stream` and before
   * later work on it. The calls of one rank write different partial slots and only read
   * their inputs, so their order does not matter. Ignored (single stream) by the decode
   * driver and whenever a call needs per-call scratch (split KV walks of short query
   * shards), which consecutive calls share. Two events are created and destroyed per
   * driver call; no device memory is allocated.
   */
  void* aux_stream;
  /*
   * 0: partial O and LSE in the two buffers described above. 1: partial_lse is not used and
   * partial_out holds one message per slot, cp_ring_message_bytes(desc) apart: the slot's O
   * (max_n_q * n_q_heads * head_dim elements of part_dtype) directly followed by its LSE
   * (max_n_q * n_q_heads floats), padded to a multiple of 256 bytes. This is the unit the
   * All2All of Algorithms 3 and 4 moves (Appendix C counts it as (D + 1) T e bytes): with
   * keep_partials in the pass-Q drivers, the N messages that rank s receives, from holders
   * k = 0..N-1 in order, are slots s * n_ranks + k, one contiguous range, and each is
   * written in place by the attention kernel and read in place by the merge: no pack,
   * permute or unpack pass.
   */
  int32_t message_layout;
  /*
   * fused_merge == 2 only. arrived: NULL (every shard is in place when the call is enqueued:
   * the single-GPU simulation), or a (host) array of n_ranks (device) pointers; arrived[k]
   * holds one int32 per ring step j of rank k, and the kernel reads the shard of step j
   * (KV of rank (k - j) mod N) only once arrived[k][j] is nonzero: whatever moves the shard
   * (a peer copy or receive on another stream) sets it afterwards. The kernel orders its
   * reads of the shard after the flag but invalidates no cache, so every step's shard needs
   * a buffer of its own that is complete before its flag is set and is not written again
   * while the kernel runs (N receive buffers per rank instead of two). The wait is bounded:
   * one thread per workgroup polls at most spin_limit (>= 1) times, a memory round trip and
   * a short sleep (a few microseconds in all) apart; if the flag stays zero the workgroup
   * leaves that shard out and sets bit j of ring_error[k] (device int32 [n_ranks], required
   * with arrived; the caller zeroes it): which steps of which ranks gave up can be read off it.
   * The outputs of such a rank are then not meaningful, but every kernel ends.
   * Limit of the contract: it relies on no line of a step's buffer being in a cache of this
   * GPU when its flag is seen. Within one launch that holds because the buffer is read only
   * after its flag. From one launch to the next (the next layer, the next call) it holds if
   * the caches are invalidated between the last read of the old contents and the arrival of
   * the new ones, which the acquire at the start of a kernel launched after the old reader
   * has finished provides; so a buffer may be reused by a later call, but not twice within
   * one launch, and not while a launch that read its old contents is still running (two walks
   * overlapping on two streams). A caller that cannot guarantee this uses a fresh buffer.
   */
  const int32_t* const* arrived;
  int32_t* ring_error;
  int32_t spin_limit;
  /*
   * Pass-Q drivers only. 1: the query shards of all ranks lie back to back in one buffer
   * (q[s + 1] == q[s] + n_q[s] rows, the same for q_pos and, for decode, bid; all n_q equal
   * and nonzero) - the small Q all-gathered instead of passed round the ring - and every KV
   * holder k answers all N steps with ONE call over the gathered queries. Requires
   * keep_partials (n_ranks * n_ranks slots), in which the partial of the queries of rank a
   * against the KV of rank b is then in slot b * n_ranks + a: the N slots a holder writes
   * are contiguous, its All2All send buffer in destination order. Not with message_layout
   * or fused_merge; CP_ERR_UNSUPPORTED if the shards are not laid out as described. 0: off.
   */
  int32_t gathered_q;
  /*
   * Prefill drivers over packed batches (the fused variable-length inputs of Algorithm 2,
   * Section 3.4), or NULL for one sequence. Not NULL: every rank's Q holds `batch` sequences
   * back to back, its share of each, with cu_seqlens_q[k] (device int32 [batch+1]) as the
   * boundaries, and its KV likewise with cu_seqlens_kv[k]; a query sees the keys of its own
   * sequence only. Each rank's share of a sequence follows the same sharding rule, so a
   * sequence shorter than 2N tokens leaves some ranks an empty segment; equal-size messages
   * are the caller's padding (CP_POS_PAD_KV / CP_POS_PAD_Q). Plain drivers only: not with
   * fused_merge, gathered_q or aux_stream.
   */
  const int32_t* const* cu_seqlens_q;
  /*
   * cp_ring_passq_decode only. 1: the caller promises that the bid arrays of all ranks
   * together name every sequence at most once (Algorithm 4: one new token per sequence), and
   * every decode call is made with CP_SHAPE_UNIQUE_BID. With gathered_q, each KV holder then
   * writes its split-KV partials into its own part of the workspace and ONE launch applies
   * Equation 4 over splits and holders together (the merge is associative, and Algorithm 4
   * merges once, after the All2All); the partial slots partial_out / partial_lse are then not
   * written. 0: no promise.
   */
  int32_t unique_bid;
} cp_ring_desc;

/* Bytes of one message of message_layout 1 (see cp_ring_desc); 0 for an invalid descriptor.
 * Host arithmetic; reads n_ranks, n_q, n_q_heads, head_dim, part_dtype. */
size_t cp_ring_message_bytes(const cp_ring_desc* desc);

/*
 * Ring pass-KV, Algorithm 2, for every virtual rank k: for j = 0..N-1,
 * s = (k - j) mod N, O_k^s = GQA(Q_k, KV^s); then O_k = merge_s(O_k^s)
 * (Equation 4). The SendRecv of the algorithm is elided: KV^s is read in place.
 */
int cp_ring_passkv(const cp_ring_desc* desc, void* stream);

/*
 * Ring pass-Q prefill, Algorithm 3: rank k computes O_s^k = GQA(Q^s, KV_k) for
 * s = (k - j) mod N; the permute + All2All that returns partials to their
 * source rank is the choice of output slot; then O_s = merge_k(O_s^k).
 */
int cp_ring_passq(const cp_ring_desc* desc, void* stream);

/*
 * Batched ring pass-Q decode, Algorithm 4: as cp_ring_passq with one query token
 * per sequence, batch ids travelling with the queries, and KV_k[bid] lookups
 * through cu_seqlens_kv[k]. Uses cp_attn_decode for every step.
 */
int cp_ring_passq_decode(const cp_ring_desc* desc, void* stream);

/* Workspace the ring drivers need: the maximum over all (query rank, KV rank) calls. */
size_t cp_ring_workspace_bytes(const cp_ring_desc* desc, int32_t decode);

/* Ring order chosen by cp_select_order. */
typedef enum { CP_ORDER_PASS_KV = 0, CP_ORDER_PASS_Q = 1 } cp_ring_order;

/* Which rule cp_select_order applies. */
typedef enum {
  CP_RULE_ANALYTIC = 0,        /* Algorithm 1 (Section 3.3): Equations 1 and 2 */
  CP_RULE_ANALYTIC_ALL2ALL = 1,/* Algorithm 5 (Appendix C): Equation 1 tightened by the All2All cost */
  CP_RULE_EMPIRICAL = 2        /* Appendix D: sign of h(T, P) = alpha ln T + beta ln(T/(T+P)) + gamma */
} cp_select_rule;

/* Model and system constants of the selection rules (host memory, read only). */
typedef struct {
  int32_t n_q_heads;      /* N_H  of the whole model (or of one GPU: only the ratio matters) */
  int32_t n_kv_heads;     /* N_KV */
  int32_t n_ranks;        /* N: CP ranks (nodes) the ring spans */
  int32_t reserved;       /* must be 0 */
  double peak_flops;      /* C: attainable attention FLOP/s of one rank */
  double bandwidth;       /* BW: bytes/s of the link that carries the ring messages */
  double bytes_per_elem;  /* e: 2 for bf16 */
  double alpha, beta, gamma; /* CP_RULE_EMPIRICAL only; all three 0 = the paper's fit
                                (-1.059, 1.145, 12.112) */
} cp_select_params;

/*
 * pass-KV or pass-Q for a prefill of t_new tokens on top of p_cached cached tokens
 * (full prefill: p_cached = 0; decode: t_new = 1). Pure host arithmetic, no GPU.
 *   CP_RULE_ANALYTIC (Algorithm 1): pass-KV iff
 *       T >= N * C * N_KV * e / (2 * N_H * BW)          (Equation 2: KV transfer hidden)
 *    or T / (T + P) >= 2 * N_KV / N_H                   (Equation 1: KV message not larger)
 *   CP_RULE_ANALYTIC_ALL2ALL (Algorithm 5): the second test becomes
 *       T / (T + P) >= 2 * N_KV / N_H - 4 * T * BW / (N * C * e).
 *   CP_RULE_EMPIRICAL (Appendix D): pass-KV iff h(T, P) > 0, natural logarithms.
 * *order_out receives a cp_ring_order. Errors: CP_ERR_NULL; CP_ERR_SHAPE for t_new < 1,
 * p_cached < 0, non-positive heads / ranks / C / BW / e; CP_ERR_UNSUPPORTED for an
 * unknown rule.
 */
int cp_select_order(const cp_select_params* params, int64_t t_new, int64_t p_cached,
                    int32_t rule, int32_t* order_out);

/*
 * Prefill with the ring order chosen at run time, as the paper's system does (Section 3.3):
 * t_new = the sum of desc->n_q, cp_select_order(params, t_new, p_cached, rule) picks
 * pass-KV or pass-Q, and the matching driver runs on `desc` (which must be valid for it; a
 * descriptor without options is valid for both). params->n_ranks must equal desc->n_ranks.
 * *order_out (host, may be NULL) receives the order taken. Errors: those of cp_select_order
 * and of the driver; CP_ERR_SHAPE if the rank counts differ or no rank has a query.
 */
int cp_ring_prefill(const cp_ring_desc* desc, const cp_select_params* params, int64_t p_cached,
                    int32_t rule, int32_t* order_out, void* stream);

/*
 * Persistent KV cache of one rank (Sections 3.5.2 and 3.6: the K/V of every turn's new tokens,
 * decode tokens included, stay in the cache of the rank that owns them and are read by the
 * later turns' partial prefill and decode).
 *
 * Layout, all device memory owned by the caller:
 *   k_cache, v_cache  [slots, n_kv_heads, head_dim] in shape->dtype, 16-byte aligned
 *   kv_pos_cache      int32 [slots]
 *   cu_seqlens_kv     int32 [batch+1]: sequence b owns slots [cu[b], cu[b+1]), its capacity
 *   seq_used          int32 [batch+1]: tokens held per sequence (they fill the front of the
 *                     sequence's slot range in arrival order), followed by one word the
 *                     library uses as a ticket counter inside cp_kv_append; it is zero
 *                     between calls
 * A slot that holds no token carries CP_POS_PAD_KV in kv_pos_cache, which no query position
 * reaches: cp_attn_decode, cp_attn_partial and the ring drivers take the cache (or one
 * sequence's slot range of it) as it is, with cu_seqlens_kv as the sequence boundaries.
 *
 * cp_kv_cache_reset marks every slot unused, clears K and V (an unused slot must not hold a
 * NaN or Inf pattern: masked keys still enter the P V product with weight zero) and zeroes
 * seq_used and *dropped (dropped may be NULL). It reads shape->dtype, head_dim, n_kv_heads,
 * batch and total_kv (= slots). Errors: CP_ERR_NULL, CP_ERR_SHAPE (batch < 1, slots negative
 * or > INT32_MAX), CP_ERR_UNSUPPORTED (dtype, head_dim), CP_ERR_ALIGN.
 */
int cp_kv_cache_reset(const cp_shape* shape, void* k_cache, void* v_cache,
                      int32_t* kv_pos_cache, int32_t* seq_used, int32_t* dropped, void* stream);

/*
 * Append new tokens to the cache described above.
 *   shape->dtype, head_dim, n_kv_heads  element type and row shape (n_q_heads is not used)
 *   shape->batch    sequences in the cache;  shape->total_kv  slots
 *   shape->total_q  number of new tokens in this call
 *   k_new, v_new    (device) [total_q, n_kv_heads, head_dim], 16-byte aligned
 *   pos_new         (device) int32 [total_q]
 *   cu_seqlens_new  (device) int32 [batch+1]: the new tokens of sequence b are rows
 *                   [cu_new[b], cu_new[b+1]); they go to slots cu_kv[b] + seq_used[b] + 0, 1, ...
 *   seq_used        (device) read, then advanced by the number of tokens taken
 *   dropped         (device) int32 or NULL: incremented by the number of tokens that did not
 *                   fit their sequence's capacity (those are not stored)
 * One launch on `stream` for small calls (up to 1024 tokens of a 256-byte row), two for
 * larger ones; calls on one cache must be ordered by the caller (same stream or events).
 * Errors: CP_ERR_NULL, CP_ERR_SHAPE, CP_ERR_UNSUPPORTED (dtype, head_dim), CP_ERR_ALIGN.
 */
int cp_kv_append(const cp_shape* shape, const void* k_new, const void* v_new,
                 const int32_t* pos_new, const int32_t* cu_seqlens_new, void* k_cache,
                 void* v_cache, int32_t* kv_pos_cache, const int32_t* cu_seqlens_kv,
                 int32_t* seq_used, int32_t* dropped, void* stream);

/*
 * Host arithmetic. Rank that takes sequence `seq`'s token (its query, and its K/V in that
 * rank's cache) at decode iteration `decode_iter`: the batch is dealt round-robin and the deal
 * moves on by one rank per iteration (Section 3.6), so every rank's cache grows at the same
 * rate. Returns the rank, or CP_ERR_SHAPE for n_ranks < 1 or a negative argument.
 */
int32_t cp_decode_owner(int32_t seq, int32_t decode_iter, int32_t n_ranks);

/* Static description of a cp_status. Never NULL. */
const char* cp_strerror(int status);

/* Library version as major * 10000 + minor * 100 + patch. */
int cp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CP_ATTN_H */
