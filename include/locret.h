/*
 * locret.h -- C ABI of the MI355X (gfx950) Locret chunk-step library.
 *
 * One attention layer's chunked-prefill step with learned KV-cache eviction
 * (arXiv 2410.01805): for every incoming chunk
 *   - attention of the chunk's queries over [retained cache ; chunk], causal inside the chunk
 *     (Section 3.1, Eq. 1, with the grouped-query head map of Section 3.1);
 *   - the retaining head  S~ = SiLU([Q,K,V] W1) W2, one score per token per KV head (Section 3.3);
 *   - stabilizer-masked top-b selection per KV head and order-preserving compaction of
 *     K, V and score into a fixed-capacity cache (Section 3.4; Appendix A.2, Algorithm 1).
 *
 * Conventions that hold for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller and must be 16-byte aligned.
 *     Only `locret_config*`, `locret_ctx**` and the out-parameters of locret_cache_view are HOST
 *     pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Compute calls only
 *     enqueue work on that stream: they never allocate, never synchronise and never read
 *     results back.  The cache length after a call is known on the host.
 *   - The workspace is allocated by the caller (locret_workspace_bytes), lent to the context
 *     for its lifetime and must not be touched while calls are in flight.
 *   - Return value: 0 (LOCRET_OK) or a negative error code.  Argument errors are found on the
 *     host before anything is launched and leave the context unchanged.
 *   - A context is not thread-safe; calls on one context must be issued in stream order.
 *
 * Layouts (row-major, innermost last; `s` = element type chosen by config.dtype)
 *   q            [T][n_q_heads][head_dim]   s    un-rotated
 *   k, v         [T][n_kv_heads][head_dim]  s    un-rotated
 *   attn_out     [T][n_q_heads][head_dim]   s
 *   scores       [n_kv_heads][T]            float
 *   kept_idx     [n_kv_heads][budget]       int32; the first n_keep entries of each row are valid
 *   W1           [d_in][d_hidden]           s
 *   W2           [d_hidden][n_kv_heads]     s
 */
#ifndef LOCRET_H
#define LOCRET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LOCRET_OK        0
#define LOCRET_EINVAL   -1   /* NULL pointer or a value outside its domain                 */
#define LOCRET_ESHAPE   -2   /* unsupported head layout / sizes, or T outside 1..chunk_max */
#define LOCRET_EALIGN   -3   /* a device pointer is not 16-byte aligned                    */
#define LOCRET_ESTATE   -4   /* call not valid in the context's state (weights missing,
                                cache would overflow its capacity)                         */
#define LOCRET_EHIP     -5   /* the HIP runtime reported an error                          */
#define LOCRET_ENOMEM   -6   /* workspace too small / host allocation failed               */
#define LOCRET_ELIMIT   -7   /* size beyond the fixed scratch of locret_score_static       */

#define LOCRET_F32   0
#define LOCRET_BF16  1

typedef struct locret_ctx locret_ctx;   /* opaque host-side handle */

/* Problem statement of Algorithm 1 (budget b, chunk size B) plus the head layout of Section 3.1. */
typedef struct {
  int32_t n_q_heads;      /* h                                                                 */
  int32_t n_kv_heads;     /* h/g; must divide n_q_heads                                        */
  int32_t head_dim;       /* d: 16, 32, 64, 96 or 128 (bf16 with 64/96/128 runs on the matrix cores) */
  int32_t chunk_max;      /* B: largest T of any call                                          */
  int32_t budget;         /* b: cache units kept per KV head                                   */
  int32_t d_hidden;       /* d_R: retaining-head hidden width (bf16: multiples of 128 run on the matrix cores) */
  int32_t rh_kv_expand;   /* 0: W1 has (h + 2 h/g) d rows, the shape Section 3.3 states
                             1: W1 has 3 h d rows; the K and V blocks are repeated g times in
                                query-head order (query head j reads KV head floor(j/g))      */
  int32_t dtype;          /* LOCRET_F32 or LOCRET_BF16: type of q, k, v, W1, W2, out and cache */
  int32_t rope_mode;      /* 0: no rotary embedding
                             1: K is cached un-rotated; at every call cache slot i is rotated to
                                position i and chunk token t (key and query) to n_c + t
                                (Section 3.4; pairs (i, i + d/2), inverse frequency theta^(-2i/d)) */
  float   rope_theta;
  float   softmax_scale;  /* 0 selects 1/sqrt(head_dim)                                        */
  int32_t kv_bits;        /* 0: the cache keeps K and V rows as given
                             4: 4-bit cache rows (appendix "Orthogonality to Other Methods", the combination
                                with 4-bit KV-cache quantization).  Every K and V row is quantized when it
                                enters the cache, per unit and per group of 32 consecutive head dims:
                                code = clamp(round-half-even((x - lo) / s), 0, 15), lo = the group's minimum,
                                s = (max - min) / 15 rounded to bf16 (1 for a constant group), in float32;
                                value = lo + code * s.  K is quantized un-rotated.  Attention (chunk and decode)
                                reads the cache, so it sees these values, the chunk's own rows included; the
                                retaining head sees the raw q, k, v.  Packed row: head_dim/2 code bytes (dim 2i
                                in the low nibble, 2i+1 in the high one), then (s, lo) as little-endian bf16 per
                                group.  Needs dtype bf16 and head_dim 64, 96 or 128 (LOCRET_ESHAPE); head-wise
                                budgets are not available with it (LOCRET_ESHAPE).  The two cache copies hold
                                packed rows only; one bf16 staging copy of the dequantized rows (K rotated)
                                serves the attention kernels.                                          */
} locret_config;

/* Bytes of device workspace a context needs (both cache copies, rotated-key shadow, score and
 * position arrays, weights in kernel layout, scratch).  0 if the config is invalid. */
size_t locret_workspace_bytes(const locret_config* cfg);

/* Validates cfg, takes the workspace (device, 256-byte aligned, >= locret_workspace_bytes) and
 * builds the rotary table.  Synchronises the device once.  *out is set only on success. */
int locret_create(const locret_config* cfg, void* dev_workspace, size_t workspace_bytes, locret_ctx** out);

/* Copies the retaining head's weights into the workspace in the layout the kernels use
 * (W1 transposed; with rh_kv_expand = 1 the g repeated row blocks are summed, which is the same
 * linear map).  W1, W2: device, layouts above.  Asynchronous on `stream`. */
int locret_set_weights(locret_ctx* ctx, const void* W1, const void* W2, void* stream);

/* Pinned prefix (Locret-Q, Section "Supporting Query-Driven Tasks": the query is placed at the start of
 * the sequence so that every eviction sees it).  From the next evicting call on, the first n_pin units
 * of the cache are kept whatever their scores, like stabilizers at the front; the rest of the budget
 * is shared as before.  Units keep their order, so once the first n_pin tokens of a stream are in the
 * cache they stay in slots 0 .. n_pin-1.  Where the last n_stab units and the prefix would overlap
 * (short lists) the stabilizers are counted first.  0 <= n_pin <= budget (LOCRET_EINVAL); an evicting
 * call with n_stab + n_pin > budget returns LOCRET_EINVAL.  Default 0; locret_reset keeps it. */
int locret_set_pinned_prefix(locret_ctx* ctx, int32_t n_pin);

/* Head-wise budgets (appendix "Orthogonality to Other Methods", head-wise budget allocation: KV heads
 * evict independently, so every head may be given a budget of its own, as PyramidKV-style allocators do).
 * budgets: HOST array of n_kv_heads values, 1 <= budgets[m] <= config.budget (LOCRET_EINVAL), copied; NULL
 * restores the single budget of the config.  Only on an empty cache (after locret_create or locret_reset;
 * LOCRET_ESTATE otherwise) and for n_kv_heads <= LOCRET_MAX_HEAD_BUDGETS (LOCRET_ESHAPE).  From then on an
 * evicting call keeps min(n_c[m] + T, budgets[m]) units of head m, so the heads' caches differ in length;
 * head m's slot i sits at position i and its chunk token t at n_c[m] + t (keys and the queries of its
 * group), the stabilizers and the pinned prefix are clamped to the head's own length, and an evicting call
 * with n_stab + n_pin > min(budgets) returns LOCRET_EINVAL.  Rows of kept_idx_out keep the stride
 * config.budget; row m holds min(n_c[m] + T, budgets[m]) entries in head m's own concatenated index space.
 * locret_reset keeps the budgets.  Host-only. */
#define LOCRET_MAX_HEAD_BUDGETS 64
int locret_set_head_budgets(locret_ctx* ctx, const int32_t* budgets);

/* Empties the cache (n_c = 0, tokens seen = 0).  Host-only. */
int locret_reset(locret_ctx* ctx);

/* The whole chunk step (Algorithm 1's loop body for one layer) for T tokens, 1 <= T <= chunk_max:
 *   attention -> attn_out; retaining head -> scores; append; if `evict` != 0: keep the last
 *   min(n_stab, n_c + T) units plus the best of the others up to `budget`, compact.
 * n_stab     stabilizer length n_s for this call, 0 <= n_stab <= budget (Algorithm 1 passes 0 on
 *            the last chunk).
 * evict      0 = append only (the trailing n_loc pass of Algorithm 1); needs n_c + T <= budget +
 *            chunk_max, else LOCRET_ESTATE.
 * scores_in  NULL, or float [n_kv_heads][T]: use these scores for the selection instead of the
 *            retaining head's (the retaining head still runs and fills scores_out).
 * scores_out NULL or float [n_kv_heads][T].
 * kept_idx_out NULL or int32 [n_kv_heads][budget]: kept indices, ascending, in the concatenated
 *            index space (i < n_c: old cache slot i; otherwise chunk token i - n_c); row m holds
 *            n_keep = min(n_c + T, budget) valid entries (all n_c + T when evict = 0 is not
 *            reported: kept_idx_out is left untouched then).
 * Selection order: score descending, then index ascending; -0 == +0; NaN below every number. */
int locret_prefill_chunk(locret_ctx* ctx, const void* q, const void* k, const void* v, int32_t T,
                         int32_t n_stab, int32_t evict, const float* scores_in, void* attn_out,
                         float* scores_out, int32_t* kept_idx_out, void* stream);

/* Decode step (Section 3.1, Eq. 1 with B = 1; the generation step that closes Algorithm 1): appends
 * ONE token at slot n_c (position n_c, like a chunk token) and attends over the n_c + 1 retained
 * units.  Never evicts: the cache grows by one unit, up to budget + chunk_max
 * (LOCRET_ESTATE beyond).
 * q [1][n_q_heads][head_dim], k, v [1][n_kv_heads][head_dim], attn_out [1][n_q_heads][head_dim]:
 *            device pointers, 16-byte aligned, un-rotated inputs, caller-owned.
 * with_score != 0: the retaining head scores the token as locret_score would, the score is stored
 *            with the unit (a later chunk step may then evict it on its merits) and copied to
 *            scores_out (NULL or float [n_kv_heads]); needs weights (LOCRET_ESTATE).
 * with_score == 0: plain generation; the unit's stored score is NaN, which the selection order
 *            ranks below every number, so a later evicting call drops such units first.
 * Asynchronous on `stream`; no allocation, no synchronisation. */
int locret_decode_step(locret_ctx* ctx, const void* q, const void* k, const void* v, int32_t with_score,
                       void* attn_out, float* scores_out, void* stream);

/* Retaining head alone (Section 3.3): scores[m][t] for T tokens; the cache is not touched. */
int locret_score(locret_ctx* ctx, const void* q, const void* k, const void* v, int32_t T,
                 float* scores, void* stream);

/* locret_score for callers that cannot allocate device memory or hand over a workspace region for scratch:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical scores, but the kernels' scratch (partial scores per block of 128 hidden units,
 * and for short chunks the partial pre-activations of a split contraction) lies in a fixed array that is
 * part of the library's device code: 20 MiB per GPU that runs the library, held until the process ends,
 * looked up once per device in locret_create.  The call allocates nothing and frees nothing.
 * Limit: blocks * n_kv_heads * T <= LOCRET_STATIC_PART_FLOATS with blocks = d_hidden / 128 on the matrix-core path
 * (bf16, d_hidden a multiple of 128) and d_hidden / 64 rounded up otherwise,
 * else LOCRET_ELIMIT and nothing is launched (the five named configurations fit at their chunk sizes).  Short
 * chunks split the contraction as locret_score does as long as the slices fit 4 Mi floats; beyond that they run
 * unsplit (same scores up to summation order).
 * Every call on a GPU, from any context, shares that GPU's array and nothing in it has to start at zero (a call
 * writes every element before reading it): calls that overlap in time on one GPU (two streams, two threads)
 * race and must be ordered by the caller.  LOCRET_ESTATE if the context was created on a device index >= 64. */
#define LOCRET_STATIC_PART_FLOATS (1u << 20)
int locret_score_static(locret_ctx* ctx, const void* q, const void* k, const void* v, int32_t T,
                        float* scores, void* stream);

/* Append + stabilizer-masked top-b + compaction alone (Section 3.4, Algorithm 1) on caller-supplied
 * scores [n_kv_heads][T]; arguments as in locret_prefill_chunk. */
int locret_evict_compact(locret_ctx* ctx, const float* chunk_scores, const void* k_chunk,
                         const void* v_chunk, int32_t T, int32_t n_stab, int32_t* kept_idx_out,
                         void* stream);

/* Units currently in the cache per KV head (the same for every head; with head-wise budgets the longest
 * head's), and tokens seen so far.  locret_cache_lens writes every head's length to lens (HOST,
 * n_kv_heads values). */
int32_t locret_cache_len(const locret_ctx* ctx);
int locret_cache_lens(const locret_ctx* ctx, int32_t* lens);
int64_t locret_tokens_seen(const locret_ctx* ctx);

/* Device pointers into the workspace for the live cache copy: K, V [n_kv_heads][row_stride][head_dim]
 * (un-rotated), score [n_kv_heads][row_stride] float, orig_pos [n_kv_heads][row_stride] int32
 * (absolute token index of each unit; bookkeeping only).  Valid until the next call that
 * evicts.  Any out-pointer may be NULL. */
int locret_cache_view(const locret_ctx* ctx, const void** K, const void** V, const float** score,
                      const int32_t** orig_pos, int32_t* len, int32_t* row_stride);

/* 4-bit rows (config.kv_bits = 4): device pointers to the live copy's packed rows, Kq, Vq
 * [n_kv_heads][row_stride][row_stride_bytes] bytes, of which the first row_bytes = head_dim/2 + 4 head_dim/32 of
 * every row are the packed row described at locret_config (the rest is padding to a multiple of 16).  With
 * kv_bits = 4 locret_cache_view returns K = NULL (no un-rotated bf16 keys exist) and V = the dequantized staging
 * values.  LOCRET_ESTATE without 4-bit rows.  Any out-pointer may be NULL. */
int locret_cache_view_q4(const locret_ctx* ctx, const void** Kq, const void** Vq, int32_t* len, int32_t* row_stride,
                         int32_t* row_bytes, int32_t* row_stride_bytes);

/* Per-stage timing for callers that measure (benchmarks, profilers).  locret_profile_enable
 * creates hipEvents for up to max_calls chunk calls (0 disables and frees them); while enabled,
 * locret_prefill_chunk records an event at each stage boundary on the call's stream (stages:
 * 0 append+rotate, 1 attention, 2 retaining head, 3 select, 4 compact).  locret_profile_read waits
 * for the recorded events, writes the summed milliseconds per stage to stage_ms (HOST, 5 doubles)
 * and the number of calls covered to *n_calls (HOST), and starts a new window.  Calls beyond
 * max_calls in one window are not recorded.
 * An event between two kernels costs a few microseconds of idle stream, so timing every stage
 * slows a step by about 3 %.  locret_profile_mode(ctx, 1) times the attention kernel only, through
 * its own dispatch (no extra packets in the stream: the step runs at full speed); the other entries
 * of stage_ms are then 0, and if the attention kernel in use cannot be timed that way *n_calls is 0.
 * Mode 0 (default) times every stage with events between the kernels.  Mode 2 times every stage through the
 * dispatches of its own kernels (first kernel's begin to last kernel's end; no extra packets, so the figures are
 * pure kernel durations, as a profiler's kernel trace reports them; where the selection rides in the attention
 * launch its entry is 0 and the attention entry covers it).  The mode can be changed while no recorded call is
 * unread (LOCRET_ESTATE otherwise). */
#define LOCRET_PROF_STAGES 5
int locret_profile_mode(locret_ctx* ctx, int32_t mode);
int locret_profile_enable(locret_ctx* ctx, int32_t max_calls);
int locret_profile_read(locret_ctx* ctx, double* stage_ms, int32_t* n_calls);

void locret_destroy(locret_ctx* ctx);

const char* locret_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LOCRET_H */
