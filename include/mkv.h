/*
 * mkv.h -- C ABI of the Moment-KV decode-step library for AMD MI355X (gfx950).
 *
 * The library owns, per (layer, sequence), the two cache pools of the paper's "Cache
 * Architecture" paragraph -- a frozen prefill pool and a budgeted decode pool -- and the
 * importance vector I, and runs Algorithm 1 ("Decoding with Moment-KV") on them with HIP
 * kernels:  append -> attention over the whole pool (Eq. 2) -> head mean of the decode slice
 * (Eq. 4) -> momentum update (Eq. 5, Eq. 6) -> capacity check (Eq. 7) -> selection of the
 * lowest-score tokens (Eq. 8) -> removal and compaction (Eq. 9).
 *
 * Conventions
 *   - every function returns MKV_OK (0) or a negative mkv_status; nothing throws or aborts, and
 *     mkv_last_error() describes the reason.  MKV_ERR_ARG, MKV_ERR_STATE, MKV_ERR_FROZEN,
 *     MKV_ERR_CAPACITY and MKV_ERR_NOMEM are found before anything is enqueued: the cache state is
 *     unchanged.  MKV_ERR_HIP from a call that changes the cache (prefill append or compression,
 *     projection, decode steps, eviction, mkv_load_decode) may come after part of its work was
 *     enqueued; the context then refuses every further call with MKV_ERR_STATE except
 *     mkv_destroy;
 *   - "device pointer" = memory of the GPU the context was created on; "host pointer" = ordinary
 *     process memory.  Each argument says which it is;
 *   - the context owns the cache memory (or borrows cfg.arena); the caller owns q/k/v/out;
 *   - all GPU work is enqueued on cfg.stream and is asynchronous, except the mkv_read_* /
 *     mkv_write_scores / mkv_load_decode calls, which synchronise that stream;
 *   - a context is not thread-safe: one caller at a time.
 *
 * Tensor element type ("storage dtype"): MKV_F32 = IEEE float, MKV_BF16 = bfloat16 (upper 16 bits
 * of a float).  Scores are always float.  All tensors are dense, row-major, last index fastest.
 * Device tensors handed to the library (q, k_new, v_new, out, k, v, x, w_k, w_v) must start on a
 * 16-byte boundary (MKV_ERR_ARG otherwise): the kernels move them in 16-byte vectors.
 */
#ifndef MKV_H
#define MKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mkv_ctx mkv_ctx;

typedef enum { MKV_F32 = 0, MKV_BF16 = 1 } mkv_dtype;

/* MKV_SCORE_LAYER_MEAN: Eq. 4 as printed -- the mean runs over all H query heads, so there is one
 * score per decode token per (layer, sequence) and a token leaves all KV heads together.
 * MKV_SCORE_PER_KV_HEAD: ablation of that reading -- one score vector per KV head, the mean running
 * over the query heads of the head's group only; every KV head then keeps its own set of decode
 * tokens (same count), chosen by its own scores. */
typedef enum { MKV_SCORE_LAYER_MEAN = 0, MKV_SCORE_PER_KV_HEAD = 1 } mkv_score_mode;

typedef enum {
  MKV_OK = 0,
  MKV_ERR_ARG = -1,       /* null pointer, index out of range, inconsistent configuration   */
  MKV_ERR_STATE = -2,     /* call not valid in the current state                             */
  MKV_ERR_FROZEN = -3,    /* prefill append after the first decode step of that sequence     */
  MKV_ERR_CAPACITY = -4,  /* prefill or decode pool would exceed its capacity                */
  MKV_ERR_NOMEM = -5,     /* device allocation failed or the given arena is too small        */
  MKV_ERR_HIP = -6        /* a HIP runtime call failed                                       */
} mkv_status;

#define MKV_NEVER_EVICT INT32_MAX

/* Parameters follow Algorithm 1's "Require" line (decoding budget B_d, momentum factor alpha)
 * plus the shapes, and two generalisations that default to the paper: evict_trigger and
 * recent_window. */
typedef struct {
  int32_t n_layers;        /* independent layers held by this context (>= 1)                     */
  int32_t batch;           /* sequences per layer (>= 1)                                         */
  int32_t n_q_heads;       /* H; multiple of n_kv_heads                                          */
  int32_t n_kv_heads;      /* Hkv; query head h reads KV head h / (H/Hkv)                        */
  int32_t head_dim;        /* D: 64 or 128                                                       */
  int32_t dtype;           /* mkv_dtype of q, k, v, out and of the cache                         */
  int32_t max_prefill;     /* capacity of the frozen pool per sequence (ragged lengths <= this)  */
  int32_t decode_budget;   /* B_d (Eq. 3, Eq. 7)                                                 */
  int32_t evict_trigger;   /* T_e >= B_d: mkv_decode_step evicts back to B_d when the decode pool
                              exceeds T_e.  T_e == B_d is the paper (Alg. 1 "if |pool_d| > B_d").
                              MKV_NEVER_EVICT: only mkv_evict evicts                            */
  int32_t decode_capacity; /* decode slots per sequence; at least evict_trigger + max(1, max_q_len), at most
                              16384; required (> B_d) with MKV_NEVER_EVICT.  0 => that least value, plus
                              -- at the paper's cadence (evict_trigger == decode_budget) on bf16 layers
                              with 128-wide heads, max_q_len 0, default attn_variant -- an eighth of the
                              budget (8..64 slots), which turns on deferred compaction: the token a step
                              evicts only has its slot marked, attention masks marked slots, and the
                              rows are compacted when the spare slots are used up (and before any
                              reader looks).  Results are those of immediate compaction; an explicit
                              decode_capacity of decode_budget + 1 keeps compaction immediate          */
  int32_t recent_window;   /* W <= B_d: the W newest decode tokens are never evicted.  0 is the
                              paper: Eq. 8 takes its candidates from the whole decode pool      */
  float   alpha;           /* momentum factor in [0, 1] (Eq. 5; the paper uses (0, 1))           */
  float   softmax_scale;   /* 0 => 1/sqrt(head_dim)                                              */
  int32_t score_mode;      /* mkv_score_mode                                                     */
  int32_t split_keys;      /* tuning: length of the key range one attention work-group takes (multiple
                              of 16, >= 64; every (sequence, KV head) unit counts 320 positions more
                              than its keys: 192 in front for the cost of starting on it, 128 behind
                              for the extra work at its end); 0 => chosen per step so that the launch
                              just fills the chip                                               */
  int32_t attn_variant;    /* tuning: attention kernel variant; 0 => library default (the
                              matrix-core kernel for bf16 x 128 layers, else the vector-ALU
                              kernel); 1..15 force variants of the latter, 16.. of the former
                              (bf16 x 128 only, else ignored)                                   */
  int32_t groups_per_cu;   /* tuning: attention work-groups per compute unit a launch aims for;
                              0 => library default                                              */
  int32_t max_q_len;       /* largest q_len mkv_decode_step_multi will be called with (1..16);
                              0 => that entry point is disabled and takes no memory.  Needs
                              MKV_BF16 and head_dim 128                                         */
  void*   stream;          /* hipStream_t, borrowed; NULL => the default stream                  */
  void*   arena;           /* optional device pointer, 256-byte aligned, caller-owned, must outlive
                              the context; NULL => the library allocates and frees              */
  size_t  arena_bytes;     /* size of arena; must be >= mkv_required_bytes(cfg)                  */
} mkv_config;

/* Device bytes a context with this configuration needs (0 if the configuration is invalid). */
size_t mkv_required_bytes(const mkv_config* cfg);

/* Validates cfg (host pointer), allocates or carves the arena, zeroes the bookkeeping.
 * *out (host pointer) receives the context.  Errors: MKV_ERR_ARG, MKV_ERR_NOMEM, MKV_ERR_HIP. */
int mkv_create(const mkv_config* cfg, mkv_ctx** out);

/* Waits for the stream, frees what the library allocated.  NULL is MKV_OK. */
int mkv_destroy(mkv_ctx* ctx);

/* Appends n_tokens prompt tokens to the prefill pool of (layer, seq) -- "Prefill Phase":
 * the prompt's K_P, V_P written to the prefill pool.  k, v: device pointers
 * [n_tokens, n_kv_heads, head_dim] in the storage dtype; copied, the caller keeps them.
 * Repeatable until that sequence's first decode step; afterwards MKV_ERR_FROZEN (the prefill pool
 * is frozen: "Cache Architecture", Eq. 3 counts it in full).  MKV_ERR_CAPACITY beyond max_prefill. */
int mkv_prefill_append(mkv_ctx* ctx, int layer, int seq, const void* k, const void* v, int n_tokens);

/* Prompt compression before decoding starts ("Integration of Moment-KV with Prefill Compression
 * Techniques": a prefill-phase method keeps a budget of prompt tokens, Moment-KV then manages the
 * decode pool).  token_scores: device pointer, float[n_prefill], the prefill method's importance
 * of every prompt token of (layer, seq) -- computing it is that method's business.  The `keep`
 * highest-scoring tokens stay, in prompt order (lowest scores leave first, the earlier token on a
 * tie), for all KV heads alike; the pool is compacted in place and its length becomes `keep`.
 * No effect if keep >= n_prefill.  MKV_ERR_FROZEN after the sequence's first decode step,
 * MKV_ERR_CAPACITY if max_prefill exceeds 16384 (the selection keeps one pool in on-chip memory). */
int mkv_prefill_compress(mkv_ctx* ctx, int layer, int seq, const float* token_scores, int keep);

/* The producer of the token that the next decode step appends (Algorithm 1, "ComputeQKV" fused
 * with the append): for every active sequence  k = RoPE(x W_k^T),  v = x W_v^T  are computed and
 * written, rounded to bf16, straight into the next free slot of the decode pool.  The decode step
 * that follows must be called with k_new = v_new = NULL for these sequences.
 *   x              device pointer [batch, hidden] bf16           the layer's input of this step
 *   w_k, w_v       device pointers [n_kv_heads*head_dim, hidden] bf16, one row per output feature
 *                  (the layout of a linear layer's weight), feature = kv_head*head_dim + i
 *   hidden         multiple of 256
 *   rope_positions device pointer int32[batch]: absolute position of the token (prompt length +
 *                  tokens generated so far, as the model counts them), 0 <= position < 2^20; the
 *                  array lives on the device, so the range is not checked, and beyond it the
 *                  short argument reduction of the rotation loses accuracy
 *   rope_theta     base of the rotary encoding.  Convention (the paper leaves positional encoding
 *                  to the model): rotate-half -- for i < head_dim/2 and angle pos*theta^(-2i/head_dim),
 *                  (k_i, k_{i+D/2}) -> (k_i cos - k_{i+D/2} sin, k_{i+D/2} cos + k_i sin); v is not rotated.
 * fp32 accumulation, the rotation in double precision.  MKV_BF16 contexts only (MKV_ERR_ARG).
 * MKV_ERR_STATE if a projected row is still waiting for its decode step; MKV_ERR_CAPACITY if an
 * active sequence has no free decode slot. */
int mkv_project_append(mkv_ctx* ctx, int layer, const void* x, const void* w_k, const void* w_v, int hidden,
                       const int32_t* rope_positions, float rope_theta, const uint8_t* seq_mask);

/* One pass of Algorithm 1 for every active sequence of one layer.
 *   q     device pointer [batch, n_q_heads, head_dim]   the step's queries
 *   k_new device pointer [batch, n_kv_heads, head_dim]  appended to the decode pool with I = 0
 *   v_new device pointer [batch, n_kv_heads, head_dim]  (both NULL: mkv_project_append has put the
 *                                                       rows in place; MKV_ERR_STATE if it has not,
 *                                                       or if it has and they are given)
 *   out   device pointer [batch, n_q_heads, head_dim]   Att_t of Eq. 2 (rows of inactive
 *                                                       sequences are left untouched)
 *   seq_mask host pointer [batch] or NULL; 0 = sequence skipped this step (no append, no update)
 * Attention runs over prefill + decode pool including the new token; the decode slice of the
 * softmax, averaged over all query heads, updates I by Eq. 5; then every active sequence whose
 * decode pool exceeds evict_trigger is evicted back to decode_budget (Eq. 7-9).
 * MKV_ERR_CAPACITY if an active sequence has no free decode slot (only with MKV_NEVER_EVICT). */
int mkv_decode_step(mkv_ctx* ctx, int layer, const void* q, const void* k_new, const void* v_new,
                    void* out, const uint8_t* seq_mask);

/* mkv_decode_step for callers that cannot allocate device memory and want none set aside per
 * context: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results, same kernels; the step's scratch (per-work-group partial results,
 * decode logits, head means, the compaction map and selection keys) lives in a static array of
 * MKV_STATIC_SCRATCH_BYTES inside the library's code object instead of the context's arena.  Every
 * GPU the library runs on holds one copy of that array until the process ends; its address is
 * looked up once per GPU (in mkv_create, else in the first call).  The call allocates nothing, on
 * the host or the device.
 *   - MKV_ERR_CAPACITY, with nothing launched, when the step's scratch would not fit; the message
 *     gives both sizes.  The need grows with batch * n_q_heads * decode_capacity (logits) and with
 *     the number of attention work-groups; the five reference workloads need 2 .. 23 MiB.
 *   - All contexts on one GPU share the array and it keeps the last call's contents.  Nothing in
 *     it has to be cleared between calls: every word a kernel of the step reads was written
 *     earlier in the same call.  Two calls that overlap in time on one GPU (different streams)
 *     race on it: keep them on one stream or order them.
 *   - mkv_read_probs after this call reads the array, so it is only valid until the next
 *     mkv_decode_step_static on that GPU.
 *   - The GPU the context was created on must be the current one (MKV_ERR_STATE otherwise): each
 *     GPU has its own copy of the array.
 *   - Under stream capture: a step's launches carry the pool sizes the host side holds at the time
 *     of the call (launch geometry, and for batches up to 32 the lengths themselves), so a captured
 *     step may only be replayed on pools of those sizes.  In steady state the sizes recur after one
 *     whole eviction cycle -- evict_trigger - decode_budget + 1 steps, or with deferred compaction
 *     the spare slots + 1 -- so capture whole cycles, with the same active sequences in every call
 *     of a cycle, and replay the graph from the state it was captured at (mkv_decode_step can be
 *     captured the same way).  No reader (mkv_read_scores, mkv_read_kv, ...) may compact a pool
 *     between two replays of a graph captured with deferred compaction; mkv_read_slots does not. */
#define MKV_STATIC_SCRATCH_BYTES (32u << 20)
int mkv_decode_step_static(mkv_ctx* ctx, int layer, const void* q, const void* k_new, const void* v_new,
                           void* out, const uint8_t* seq_mask);

/* q_len decode steps of every active sequence in one pass over the cache (chunked or speculative
 * decoding): the result equals q_len consecutive mkv_decode_step calls whose capacity check is
 * held back until the last of them.
 *   q     device pointer [batch, q_len, n_q_heads, head_dim]
 *   k_new device pointer [batch, q_len, n_kv_heads, head_dim]  appended in order, each with I = 0
 *   v_new device pointer [batch, q_len, n_kv_heads, head_dim]
 *   out   device pointer [batch, q_len, n_q_heads, head_dim]   Att of Eq. 2 per query row
 * Query row i attends to the prefill pool, the decode pool and the appended tokens 0..i (Eq. 2 over
 * the pool as it stands at that step).  The scores take q_len momentum updates in row order
 * (Eq. 4, Eq. 5), an appended token starting at I = 0 in its own step (Eq. 6); then every active
 * sequence whose decode pool exceeds evict_trigger is evicted back to decode_budget (Eq. 7-9).
 * Needs cfg.max_q_len >= q_len >= 1 (else MKV_ERR_ARG; MKV_ERR_STATE when max_q_len is 0).
 * MKV_ERR_CAPACITY if an active sequence has fewer than q_len free decode slots. */
int mkv_decode_step_multi(mkv_ctx* ctx, int layer, int q_len, const void* q, const void* k_new,
                          const void* v_new, void* out, const uint8_t* seq_mask);

/* Capacity enforcement on demand (Eq. 7-9): every selected sequence whose decode pool exceeds
 * decode_budget loses its overflow lowest-score tokens outside the recent window -- ties go to
 * the older token -- and the survivors' K, V, score and position rows are compacted in order of
 * generation.  seq = -1: all sequences of the layer.  MKV_OK and no effect when within budget. */
int mkv_evict(mkv_ctx* ctx, int layer, int seq);

/* Reads the importance vector (Eq. 5) and the original decode positions of (layer, seq) into host
 * buffers of `capacity` entries; *n_out = decode pool size.  Either buffer may be NULL.
 * MKV_ERR_CAPACITY if capacity is too small. */
int mkv_read_scores(mkv_ctx* ctx, int layer, int seq, float* scores, int32_t* positions,
                    int capacity, int* n_out);

/* ---- parity / snapshot helpers (not on the hot path) ---------------------------------------- */

/* Overwrites the first n scores of (layer, seq) from a host buffer; n must equal the pool size. */
int mkv_write_scores(mkv_ctx* ctx, int layer, int seq, const float* scores, int n);

/* Restores a decode pool: k, v device pointers [n, n_kv_heads, head_dim]; scores, positions host
 * pointers [n] (positions strictly increasing, all < next_step).  Replaces the decode pool of
 * (layer, seq), sets its step counter to next_step and freezes its prefill pool. */
int mkv_load_decode(mkv_ctx* ctx, int layer, int seq, const void* k, const void* v,
                    const float* scores, const int32_t* positions, int n, int64_t next_step);

/* Copies one KV head of a pool to host buffers [n, head_dim] (storage dtype).
 * pool: 0 = decode pool, 1 = prefill pool.  Either buffer may be NULL. */
int mkv_read_kv(mkv_ctx* ctx, int layer, int seq, int pool, int kv_head, void* k, void* v,
                int capacity, int* n_out);

/* After mkv_decode_step(layer): the head-mean decode-slice attention abar (Eq. 4) the step added
 * to the scores, for the pool as it was before that step's eviction (host float[capacity]), and the
 * natural-log softmax normaliser per query head (host float[n_q_heads]).  Either may be NULL.
 * After mkv_decode_step_multi: the same two for its last query row.
 * MKV_ERR_STATE if `layer` was not the layer stepped last. */
int mkv_read_probs(mkv_ctx* ctx, int layer, int seq, float* abar, float* lse_per_head,
                   int capacity, int* n_out);

/* The decode pool of (layer, seq) slot by slot, without compacting it (with deferred compaction the
 * other readers close the holes first): scores and original positions per slot (host float /
 * int32 [capacity]), live[j] = 0 where slot j holds a token that has been evicted and awaits
 * compaction (host uint8 [capacity]); *n_slots = slots in use; *pending_slot = the slot the last
 * decode step selected for eviction and that is still marked live, or -1.  Any pointer may be NULL.
 * A context without deferred compaction reports every slot live and nothing pending. */
int mkv_read_slots(mkv_ctx* ctx, int layer, int seq, float* scores, int32_t* positions, uint8_t* live,
                   int capacity, int* n_slots, int* pending_slot);

/* MKV_SCORE_PER_KV_HEAD only: selects the KV head whose score vector mkv_read_scores,
 * mkv_write_scores and mkv_read_probs (abar) address from now on (default 0).  mkv_load_decode
 * gives every head the same scores and positions.  MKV_ERR_ARG outside [0, n_kv_heads), and for
 * anything but 0 in MKV_SCORE_LAYER_MEAN mode. */
int mkv_set_score_view(mkv_ctx* ctx, int kv_head);

/* Host-side bookkeeping of (layer, seq): prefill length, decode pool size, decode steps taken. */
int mkv_get_lens(mkv_ctx* ctx, int layer, int seq, int* n_prefill, int* n_decode, int64_t* step);

/* ---- measurement helper (off by default) ---------------------------------------------------- */

/* enable != 0: every following mkv_decode_step launches its attention kernel, its finishing
 * kernel and its eviction kernels with start/stop HIP events attached to the launch itself, so the
 * recorded times are the kernels' own execution times on the context's stream (the events slow
 * the step a little: use a separate pass for whole-step timing).  enable == 0 stops recording.
 * Either way the accumulated figures are reset. */
int mkv_set_profiling(mkv_ctx* ctx, int enable);

/* Waits for the stream and returns the sums since mkv_set_profiling: microseconds spent in the
 * attention, finishing and eviction kernels (host pointers to 3 doubles) and the number of steps
 * and of steps that evicted (host pointers to 2 int64).  Any pointer may be NULL. */
int mkv_read_profile(mkv_ctx* ctx, double* kernel_us, int64_t* counts);

/* Text of the last error on this context (or of the last failed mkv_create when ctx is NULL). */
const char* mkv_last_error(const mkv_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* MKV_H */
