/*
 * tkv -- tiered KV-cache decode attention for one MI355X (gfx950).
 *
 * C ABI of the per-decode-step hot path of "Not All Thoughts Need HBM: Semantics-Aware Memory
 * Hierarchy for LLM Reasoning": grouped-query decode attention over a four-tier KV cache
 * (Sec. 3.2: T0 resident in HBM, T1 kept at full precision in host DDR and prefetched, T2 held
 * compressed and dequantised inside the kernel, T3 evicted and skipped), the cumulative
 * per-position importance score accumulated by the same pass (Sec. 3.1, Eq. 1), the rank-based
 * tier assignment of Sec. 3.3 / Algorithm 1, and the row movement between tiers (Algorithm 1,
 * "offload" / "trim"; Sec. 3.4 prefetching).
 *
 * Conventions
 *  - Every call returns a tkv_status (0 = OK, negative = error); nothing throws or aborts.
 *    tkv_last_error() returns a NUL-terminated message owned by the handle (or a static string
 *    when the handle is NULL); it stays valid until the next failing call on that handle.
 *  - "device" pointers are HIP device addresses on config.device; "host" pointers are ordinary
 *    host memory.  Buffers passed in are caller-owned and only borrowed until the work enqueued
 *    by the call has completed on `hip_stream`.  Everything the library allocates (pools, index
 *    lists, the pinned T1 store, side streams, events) is library-owned and released by tkv_destroy.
 *  - Device and pinned-host memory is obtained through the allocator callbacks of tkv_config
 *    (hipMalloc / hipHostMalloc when they are NULL).
 *  - `hip_stream` is a hipStream_t (NULL = the default stream).  tkv_append and
 *    tkv_attend_and_score only enqueue work and return; tkv_classify and tkv_migrate enqueue work
 *    and read a few counters back (one short synchronisation each); the tkv_get_ / tkv_set_ calls
 *    synchronise.  All calls on one handle must come from one thread at a time and use one stream.
 *  - All sequences of a handle have the same length; a layer's length is the number of tokens
 *    appended to it.  One tier and one score exist per (sequence, position), shared by all layers
 *    and kv heads (Algorithm 1 moves positions, not per-layer rows).
 *  - Inputs must be finite; scores are non-negative.
 */
#ifndef TKV_H
#define TKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tkv_cache tkv_cache;

typedef enum {
  TKV_OK = 0,
  TKV_EINVAL = -1,    /* bad argument or configuration */
  TKV_ENOMEM = -2,    /* an allocator callback returned NULL */
  TKV_ECAPACITY = -3, /* a pool, the host store or max_tokens would overflow; state unchanged */
  TKV_ESTATE = -4,    /* call not valid in the current state (e.g. layers of unequal length) */
  TKV_EDEVICE = -5    /* a HIP call failed */
} tkv_status;

typedef enum { TKV_F32 = 0, TKV_BF16 = 1, TKV_F16 = 2 } tkv_dtype;   /* binary32, bfloat16, binary16 */

/* T2 encodings (Sec. 3.2 only says "reduced precision, e.g. 8-bit"); both are symmetric, defined in
 * IEEE binary32 with round-to-nearest-even and true division, K row and V row encoded separately:
 *  INT8_ROW: per row a = max|x|, scale = a/127 (binary32), code = clamp(rne(x/scale), -127, 127);
 *  INT4_G32: groups of 32 along head_dim, scale = binary16_rne(a/7), code = clamp(rne(x/scale), -7, 7),
 *            two codes per byte (element 2j in the low nibble, two's complement).
 * A zero scale gives zero codes.  x_hat = code * scale. */
typedef enum { TKV_T2_INT8_ROW = 0, TKV_T2_INT4_G32 = 1 } tkv_t2_format;

/* How attention is ordered against the T1 prefetch of a layer after a tkv_migrate (Sec. 3.4):
 *  WAIT: the first tkv_attend_and_score of a layer waits (on the GPU, event-ordered) until that layer's
 *        newly offloaded rows have made the trip device -> pinned host -> staging buffer;
 *  LAZY: attention keeps reading such rows from their old HBM slot until the staged copy has arrived
 *        (polled without blocking) and then switches; outputs are bit-identical either way (Prop. 1).
 *  STREAM: T1 rows are not kept in HBM at all between uses: the staging buffer is two layer-sized frames shared by
 *        all layers, and every tkv_attend_and_score reads its layer's T1 rows from a frame that was refilled from the
 *        pinned store (hipMemcpyAsync on the prefetch stream, event-ordered) while the previous layers were attended.
 *        HBM then holds T0, T2 and two frames; every decode step moves all of T1 over the host link (and the rows of
 *        the pinned store whose positions have left T1 since the store was last rewritten; tkv_migrate rewrites it
 *        packed, beside the frame pass it makes anyway, when those rows would cost more link time until the next
 *        plan than the rewrite).
 *        STREAM is the one mode that does NOT promise Prop. 1's bit identity: the T1 rows of a layer are served by a
 *        second launch over the frame, with tiles and splits of its own, so the binary32 summation order depends on
 *        which rows are in T1.  Row bits are still exact (the T1 rows attended are the rows appended), and outputs and
 *        scores agree with the all-in-HBM placement to binary32 rounding (a few 1e-7 relative), far inside the
 *        tolerances of the method; only bit equality is given up. */
typedef enum { TKV_PREFETCH_WAIT = 0, TKV_PREFETCH_LAZY = 1, TKV_PREFETCH_STREAM = 2 } tkv_prefetch_mode;

/* What a layer call adds to the cumulative score of a position:
 *  ATTENTION: score_scale * sum over query heads of the attention weight (Eq. 1; the paper's method);
 *  VATP: the value-aware variant of the paper's scoring ablation (Sec. "Ablation: Importance Scoring Methods"): each
 *        head's weight is multiplied by the Euclidean norm of the value row that head reads at the position.  The norm
 *        is taken once, from the row as appended (binary32, fixed summation order); it does not follow the row
 *        through later compression.  Costs 4 bytes per (layer, sequence, kv head, position) of device memory.
 *  REDUNDANCY: "attn - redundancy" of the same ablation.  The paper gives no formula for the redundancy term; this
 *        library's reading: rho of a position in a (layer, kv head) is the cosine similarity of its key row with the key
 *        row appended just before it, clamped below at 0 (0 for the first position or an all-zero row), taken once from
 *        the rows as appended.  Per query head a layer call adds the attention weight minus
 *        redundancy_weight * rho / (positions the query attends to); evicted positions receive nothing.  Scores can go
 *        below zero; tkv_classify ranks binary32 scores by value.  Costs 4 bytes per (layer, sequence, kv head,
 *        position) plus one key row per (layer, sequence, kv head).
 *  COMBINED: "attn x val - redundancy": the VATP term minus the same penalty (both arrays). */
typedef enum { TKV_SCORE_ATTENTION = 0, TKV_SCORE_VATP = 1, TKV_SCORE_REDUNDANCY = 2, TKV_SCORE_COMBINED = 3 } tkv_scorer;

typedef struct {
  int32_t n_layers, batch, n_q_heads, n_kv_heads, head_dim; /* head_dim in {64, 128}; n_q_heads % n_kv_heads == 0,
                                                               group size n_q_heads / n_kv_heads <= 8 */
  int32_t max_tokens;                  /* per-sequence capacity in positions (< 2^24) */
  int32_t kv_dtype;                    /* tkv_dtype: type of K, V and q */
  int32_t out_dtype;                   /* tkv_dtype of the attention output.  binary32 keeps the accumulator's value;
                                          bf16 / binary16 add one round-to-nearest-even (up to 2^-8 / 2^-11 relative
                                          per element) */
  int32_t t2_format;                   /* tkv_t2_format */
  int32_t n_prompt, k_sink, k_window;  /* protected regions (Sec. 3.2): prompt, first k_sink reasoning tokens,
                                          last k_window tokens; never offloaded, compressed or evicted */
  float score_scale;                   /* factor on the per-layer sum over query heads; 0 -> 1/(n_layers*n_q_heads) (Eq. 1) */
  float softmax_scale;                 /* 0 -> 1/sqrt(head_dim) (Eq. 3) */
  int32_t t0_rows, staging_rows, t2_rows; /* per-sequence capacity (in positions) of the HBM pool, the T1 staging
                                          buffer and the compressed pool; 0 -> max_tokens.  The staging buffer exists
                                          once per layer, or (TKV_PREFETCH_STREAM) as two frames for all layers.  A migrate
                                          takes the slots of the rows that enter a pool before it releases those of the
                                          rows that leave it, so a pool needs room for one plan's set plus its entrants */
  int64_t host_rows;                   /* capacity of the pinned T1 store in positions, all sequences; 0 -> batch*max_tokens.
                                          Rows are handed out in order; when they run out tkv_migrate rewrites the store with
                                          the rows T1 holds at that moment (one full D2H of T1), so it must hold the T1 set
                                          of one plan plus the rows entering it, not the history of all plans */
  int64_t bounce_bytes;                /* size of each of the two device bounce rings used for T1 traffic; 0 -> 64 MiB */
  int32_t prefetch_mode;               /* tkv_prefetch_mode */
  int32_t profile;                     /* bit 0: time every attention kernel with HIP events; bit 1: time every
                                          tkv_decode_step with one pair of HIP events (tkv_get_stats) */
  int32_t scorer;                      /* tkv_scorer */
  int32_t device;                      /* HIP device ordinal */
  float redundancy_weight;             /* weight of the redundancy penalty (REDUNDANCY, COMBINED); 0 -> 1 */
  void* (*dev_alloc)(size_t bytes, void* ctx); /* device memory, 256-byte aligned; NULL -> hipMalloc */
  void (*dev_free)(void* p, void* ctx);
  void* (*pin_alloc)(size_t bytes, void* ctx); /* pinned host memory; NULL -> hipHostMalloc */
  void (*pin_free)(void* p, void* ctx);
  void* alloc_ctx;
} tkv_config;

/* Band sizes as parts per million; the four fractions must sum to 1 000 000.
 * count_rule TKV_COUNT_TOTAL (0): fractions of the whole candidate set U (non-protected positions, evicted ones
 *   included): n3, n2, n0 are floors, T1 takes the remainder; positions evicted earlier count towards n3, so the
 *   evicted share stays at f3 however many events there are (Sec. 3.3 "bottom r_evict %").
 * count_rule TKV_COUNT_ALG1 (1): Algorithm 1 as printed, which evicts again at every event: of the `live` candidates
 *   still in the cache floor(f3 * live) more are evicted, and of the s survivors floor(f0/(1-f3) * s) stay in HBM,
 *   floor(f2/(1-f3) * s) are compressed, the rest goes to T1.  With f3 = r, f0 = beta*(1-r), f2 = 0 these are
 *   n_evict = floor(r|U|), n_hbm = floor(beta(|U| - n_evict)) of Algorithm 1. */
typedef enum { TKV_COUNT_TOTAL = 0, TKV_COUNT_ALG1 = 1 } tkv_count_rule;
typedef struct { uint32_t f_t0_ppm, f_t1_ppm, f_t2_ppm, f_t3_ppm; uint32_t count_rule; } tkv_policy;

typedef struct {
  int64_t tier_count[4];      /* positions per tier, summed over sequences */
  int64_t h2d_bytes, d2h_bytes; /* T1 traffic over the host link since creation */
  int64_t h2d_copies, d2h_copies;
  double h2d_ms, d2h_ms;      /* event-timed busy time of those copies */
  double attn_kernel_ms;      /* profile != 0: summed duration of the attention kernels (the dominant kernel of a call) */
  int64_t attn_kernel_launches;
  double classify_ms, migrate_ms; /* host wall time spent inside the calls */
  int64_t attend_waits;       /* WAIT mode: attention calls that were ordered behind a prefetch event */
  int64_t lazy_old_reads;     /* LAZY mode: attention calls that still read pre-offload slots */
  int64_t n_classify, n_migrate;
  int64_t n_rehome;           /* times the pinned T1 store ran full and was rewritten, packed, from the staged copies */
  int64_t host_rows_used;     /* rows of the pinned T1 store handed out since the last rewrite (all sequences) */
  int64_t n_repack;           /* streamed T1: plans during which the store was rewritten packed because its stale rows
                                 (positions no longer in T1) would have cost more link time than the rewrite */
  int64_t device_bytes;       /* device memory the cache holds (pools, frames, lists, scratch) */
  int64_t pinned_bytes;       /* pinned host memory the cache holds */
  double attn_finish_ms;      /* profile != 0: summed duration of the finishing kernels (merge, output, scores) */
  double attn_call_ms;        /* profile bit 0: summed time from the start of a call's first kernel to the end of its last
                                 (the event pairs around every kernel stretch the gaps between them) */
  double step_ms;             /* profile bit 1: summed device time of the tkv_decode_step calls, from an event before the
                                 append launch to one behind the last layer's finishing kernel */
  int64_t steps_timed;
} tkv_stats;

/* ---- life cycle ------------------------------------------------------------------------------ */
/* Validates cfg (host memory), allocates all pools; *out receives the handle.  EINVAL / ENOMEM / EDEVICE. */
tkv_status tkv_create(const tkv_config* cfg, tkv_cache** out);
/* Waits for outstanding work, frees everything.  NULL is allowed. */
void tkv_destroy(tkv_cache* c);

/* ---- the hot path ------------------------------------------------------------------------------ */
/* Algorithm 1: the cache grows by the generated token(s).  k, v: device, [batch, n_new, n_kv_heads, head_dim]
 * in kv_dtype.  The new positions enter T0 (they are inside the recent window).  ECAPACITY beyond
 * max_tokens or the HBM pool; ESTATE while a tier plan is pending (classified or set, not yet migrated) or if
 * the new range would only partly overlap positions another layer has already appended. */
tkv_status tkv_append(tkv_cache* c, int32_t layer, const void* k, const void* v, int32_t n_new, void* hip_stream);

/* Eq. 2-3 and Eq. 1 for one layer: q device [batch, n_q_heads, head_dim] kv_dtype; out device, same shape, in
 * out_dtype.  out_h = sum over live positions of softmax(q_h . k_i * softmax_scale) v_i with kv head h / G; evicted
 * positions are skipped and the softmax renormalises over the rest; T2 rows enter as code*scale.  Adds
 * score_scale * sum over all query heads of the weights to score[b, i] for every live position.
 * A sequence whose positions are all evicted (only a forced plan can do that) gets an all-zero output and no score
 * update.  ESTATE on an empty layer. */
tkv_status tkv_attend_and_score(tkv_cache* c, int32_t layer, const void* q, void* out, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same call as tkv_attend_and_score, same arguments, same bits in out and in the scores, but the
 * call's scratch (scaled logits, split partials) lives in a fixed 16 MiB array in the library's device image instead
 * of the handle's own allocations, and the call itself makes no hipMalloc / hipFree / event or stream creation and
 * issues none of the T1 copies a TKV_PREFETCH_LAZY migrate has left queued (rows still in flight are read from their
 * old HBM slots, which by Prop. 1 gives the same bits; the next ordinary call issues the copies).
 * ECAPACITY, with the sizes in tkv_last_error, if the cache's shape needs more scratch than the array holds
 * (batch * n_q_heads * (max_tokens + 192) * 4 bytes of logits plus the partials); EINVAL with TKV_PREFETCH_STREAM.
 * All calls on one GPU share that GPU's array and it keeps the last call's contents: calls that overlap on one GPU
 * (two handles on two streams) race; calls ordered on one stream do not, and nothing in it has to start at zero. */
tkv_status tkv_attend_and_score_noalloc(tkv_cache* c, int32_t layer, const void* q, void* out, void* hip_stream);

/* The same for n_q query tokens per sequence at once (a chunk of drafted or prompt tokens whose rows have been
 * appended): q device [batch, n_q, n_q_heads, head_dim], out the same shape.  Query j belongs to position
 * n - n_q + j of the layer's n positions and attends to the positions up to and including its own (Eq. 2 sums
 * i = 1..t for the token at t); each query adds its weights to the scores (Eq. 1), in the order j = 0 .. n_q-1, which
 * is what n_q single-token steps would have done.  With 16-bit rows the tokens of a chunk ride as extra columns of
 * one launch (up to 32 / group size of them, at most 16; longer chunks go in groups), so the cache is read once per
 * group; the first call allocates scratch for one such group from the handle's allocator.  binary32 rows and
 * TKV_PREFETCH_STREAM take the decode kernels once per token.  Outputs and scores agree with single-token steps to
 * binary32 rounding (the summation order differs), not bit for bit; T1 placement stays bit-invisible (Prop. 1).
 * ESTATE unless all n_q positions were appended after the last tkv_migrate (they are then in T0). */
tkv_status tkv_attend_and_score_chunk(tkv_cache* c, int32_t layer, const void* q, void* out, int32_t n_q, void* hip_stream);

/* One decode step of Algorithm 1's loop body for all layers, in layer order: for every layer l,
 * tkv_append(l, k_all[l], v_all[l], 1) then tkv_attend_and_score(l, q_all[l], out_all[l]).  Device pointers:
 * k_all, v_all [n_layers, batch, 1, n_kv_heads, head_dim] kv_dtype; q_all [n_layers, batch, n_q_heads, head_dim]
 * kv_dtype; out_all [n_layers, batch, n_q_heads, head_dim] out_dtype.  Same errors as the two calls.  All capacity and
 * state checks are made before anything is enqueued; when all layers are at the same length the new rows of every
 * layer go in with one launch, so a later failure at layer l (a HIP error) leaves the step's rows appended to ALL
 * layers and only layers < l attended: finish the step with tkv_attend_and_score for layers >= l, or destroy the handle. */
tkv_status tkv_decode_step(tkv_cache* c, const void* k_all, const void* v_all, const void* q_all, void* out_all,
                           void* hip_stream);

/* Sec. 3.3 / Algorithm 1 "tier management", device only: ranks the candidates of every sequence by
 * (already evicted first, score bits, position) and writes the pending tier array; no KV row moves.
 * ESTATE if layers differ in length; EINVAL if the policy does not sum to 10^6. */
tkv_status tkv_classify(tkv_cache* c, const tkv_policy* policy, void* hip_stream);

/* Applies the pending tier array (from tkv_classify or tkv_set_tiers): compacts the per-tier index lists,
 * T0->T1 rows go device -> pinned host store -> staging buffer on side streams (bits preserved), T1->T0 rows
 * are copied back inside HBM, rows entering T2 are encoded from their current stored value, rows leaving T2
 * are stored as binary32(code*scale) rounded to kv_dtype, T2->T2 keeps its codes, rows entering T3 are
 * dropped everywhere.  ESTATE without a pending plan or if a position would leave T3; ECAPACITY if a pool
 * cannot take the rows entering it (nothing is changed then).
 * TKV_PREFETCH_STREAM: T0->T1 rows only make the trip to the pinned store; rows leaving T1 for T0 or T2 are read
 * back from it through the frames, layer by layer, inside this call. */
tkv_status tkv_migrate(tkv_cache* c, void* hip_stream);

/* ---- inspection and test hooks (host pointers; these synchronise) -------------------------- */
tkv_status tkv_get_scores(tkv_cache* c, float* host_out /* [batch, max_tokens] */);
tkv_status tkv_set_scores(tkv_cache* c, const float* host_in /* [batch, max_tokens], >= 0 */);
tkv_status tkv_get_tiers(tkv_cache* c, uint8_t* host_out /* [batch, max_tokens], current tiers */);
tkv_status tkv_get_pending_tiers(tkv_cache* c, uint8_t* host_out /* [batch, max_tokens]; ESTATE if none */);
/* Forces a plan (teacher forcing, invariant tests); apply it with tkv_migrate. */
tkv_status tkv_set_tiers(tkv_cache* c, const uint8_t* host_in /* [batch, max_tokens] */);
/* Ascending positions of one tier of one sequence; host_out holds max_tokens entries. */
tkv_status tkv_get_index_list(tkv_cache* c, int32_t tier, int32_t seq, int32_t* host_out, int32_t* count);
/* Codes and scales of one T2 row.  INT8_ROW: codes int8[head_dim], scales float[1];
 * INT4_G32: codes uint8[head_dim/2], scales uint16 (binary16 bits)[head_dim/32].  which: 0 = K row, 1 = V row. */
tkv_status tkv_get_t2_row(tkv_cache* c, int32_t layer, int32_t seq, int32_t kv_head, int32_t pos, int32_t which,
                          void* host_codes, void* host_scales);
/* The stored full-precision row of a T0/T1 position (kv_dtype, head_dim elements), read from where it
 * currently lives (HBM pool, or the pinned host store for T1).  ESTATE for T2/T3 positions. */
tkv_status tkv_get_row(tkv_cache* c, int32_t layer, int32_t seq, int32_t kv_head, int32_t pos, int32_t which,
                       void* host_out);
/* Blocks until every T1 transfer started by tkv_migrate (and, TKV_PREFETCH_STREAM, every frame refill in flight) has
 * landed. */
tkv_status tkv_wait_prefetch(tkv_cache* c);
tkv_status tkv_get_stats(tkv_cache* c, tkv_stats* out);
/* Sets the timing bits of tkv_config.profile (0: off, 1: per kernel, 2: per decode step, 3: both). */
tkv_status tkv_set_profile(tkv_cache* c, int32_t on);
/* Measurement helper (no cache needed): streams `bytes` of device memory through a read-only kernel with the attention
 * kernel's launch shape (one 512-lane workgroup per compute unit, 16-byte loads), iters times after one warm-up pass, on
 * the current device; *ms_per_pass (host) receives the average kernel time from the dispatch's own timestamps.  What a
 * launch of that size can reach on this GPU at best: the yardstick next to the published peak. */
tkv_status tkv_probe_hbm_read(const void* device_buf, size_t bytes, int32_t iters, void* hip_stream, float* ms_per_pass);
int32_t tkv_layer_length(const tkv_cache* c, int32_t layer); /* -1 on bad arguments */
const char* tkv_last_error(const tkv_cache* c);

/* Pure host helper: band sizes (n0, n1, n2, n3) among m candidates of which n_already_evicted are already in
 * T3 (those never come back; under TKV_COUNT_TOTAL a surplus is taken from n2, then n1, then n0).  EINVAL on a
 * bad policy. */
tkv_status tkv_tier_counts(const tkv_policy* policy, int64_t m, int64_t n_already_evicted, int64_t out[4]);

#ifdef __cplusplus
}
#endif
#endif /* TKV_H */
