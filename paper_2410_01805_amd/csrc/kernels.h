// Internal launch interface between the C-ABI host code (api.hip) and the gfx950 kernels.
// Not part of the public boundary (include/locret.h is).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace locret {

// Optional pair of events a launcher attaches to its dominant kernel's own dispatch
// (hipExtLaunchKernelGGL): the kernel's begin and end are time-stamped without separate event
// packets in the stream, which each cost a few microseconds of bubble.  Null = plain launch.
struct LaunchTimer {
  hipEvent_t start = nullptr;
  hipEvent_t stop = nullptr;
};

// Stage timer for the launchers that take no LaunchTimer.  While the host code has one set (around one stage of a
// step, on the calling thread), every launch made through launch_kernel goes out with events attached to its own
// dispatch: `start` with the first launch of the stage only, `stop` with each (the last launch's is the one
// read).  Null: plain launches.
struct StageTimer {
  hipEvent_t start = nullptr;
  hipEvent_t stop = nullptr;
  int launches = 0;
};
extern thread_local StageTimer* tl_stage_timer;

template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem, hipStream_t st, Args... args) {
  StageTimer* t = tl_stage_timer;
  if (t) {
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)shmem, st, t->launches == 0 ? t->start : nullptr, t->stop, 0,
                          static_cast<KArgs>(args)...);
    t->launches++;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, shmem, st, static_cast<KArgs>(args)...);
  }
}

// Head-wise budgets (appendix "Orthogonality to Other Methods", head-wise budget allocation: KV heads evict
// independently, so each may have its own budget): the heads' caches then differ in length.  Kernels take
// this by value beside the common length; ragged == 0: every head has the common length.
constexpr int MAX_HEAD_BUDGETS = 64;
struct HeadLens {
  int ragged;
  int v[MAX_HEAD_BUDGETS];
};
__host__ __device__ inline int head_len(const HeadLens& hl, int m, int common) { return hl.ragged ? hl.v[m] : common; }
inline HeadLens head_lens_or_common(const HeadLens* hl) {
  HeadLens r;
  if (hl) r = *hl; else r.ragged = 0;
  return r;
}

// KV heads from the longest cache to the shortest (ties: lower head first), for launches that hand out
// the long heads' work first.
struct HeadOrder {
  unsigned char v[MAX_HEAD_BUDGETS];
};
inline HeadOrder longest_first(const HeadLens& hl, int h_kv) {
  HeadOrder o;
  for (int m = 0; m < MAX_HEAD_BUDGETS; ++m) o.v[m] = (unsigned char)m;
  if (!hl.ragged) return o;
  for (int i = 1; i < h_kv; ++i) {             // insertion sort: stable, h_kv <= 64
    const unsigned char x = o.v[i];
    int j = i;
    for (; j > 0 && hl.v[o.v[j - 1]] < hl.v[x]; --j) o.v[j] = o.v[j - 1];
    o.v[j] = x;
  }
  return o;
}

// One selection (Section 3.4 and Algorithm 1: stabilizer mask, then top-b) for every KV head: scores S[m][cap],
// units [0, L), n_keep kept per head = the first n_pin units, the best of the middle ones, the last n_stab.
struct SelectArgs {
  const float* S;
  int cap, L, n_keep, n_stab, n_pin;
  int32_t* kept;        // [h_kv][kept_stride] ascending unit indices
  int kept_stride;
  int32_t* kept2;       // optional second copy (caller's buffer), or NULL
  int stride2;
  // Optional first step (register-resident form inside the attention launch only): sum the retaining
  // head's partial scores part[p][m][t], p < n_parts in ascending order, into S_w[m][L - red_T + t] (the rows
  // of S that the selection then reads) and red_out[m][t]; part == NULL: the scores are already in S.
  const float* part;
  int n_parts, part_T, h_kv, red_T;
  float* S_w;
  float* red_out;
  // Head-wise budgets: L and n_keep per head (ragged == 0: the scalars above); n_stab and n_pin are then the
  // requested lengths and every head clamps them to its own L: n_stab' = min(n_stab, L), n_pin' = min(n_pin,
  // L - n_stab').
  HeadLens L_h, keep_h;
};

// Launch switches for tests and measurements.  Read from the environment when a context is sized and created
// (LOCRET_ATTN_VARIANT, LOCRET_PP_SPLIT, LOCRET_PP_SPREAD, LOCRET_SCORE_SPLIT, LOCRET_DEC_KEYS,
// LOCRET_FUSE_SELECT), and carried with the context's dimensions; no launch path reads the environment.
struct Tuning {
  int attn_regstaged = 0;   // 1: the register-staged attention kernel also where the direct-to-LDS one applies
  int pp_split = -1;        // key ranges per item of the direct-to-LDS attention kernel: -1 chosen per launch, 0 never, k always k
  int score_nt = 0;         // retaining head: tokens per workgroup (0: by the chunk length, 64, 128)
  int pp_spread = -1;       // its workgroup order: -1 by head lengths, 0 one KV head per XCD, 1 every head over all XCDs
  int score_split = -1;     // contraction slices of the retaining head: -1 chosen per launch, 0 never, k always k
  int dec_keys = 0;         // keys per split of the decode step: 0 chosen per launch, else a multiple of 64 in 64..65536
  int fuse_select = 1;      // 0: the selection is always a launch of its own
};

struct Dims {
  Tuning tune;
  int h;        // query heads
  int h_kv;     // KV heads
  int g;        // h / h_kv
  int d;        // head dim
  int cap;      // rows per KV head in every cache array (budget + chunk_max)
  int bf16;     // 0: float storage, 1: bf16 storage
  int rope;     // rotary mode
  int K;        // retaining-head input width after folding: (h + 2 h_kv) d
  int d_R;      // retaining-head hidden width
  int kv_bits;  // 0: cache rows in the storage type; 4: packed 4-bit rows plus one bf16 staging copy (quant_rows.hip)
};

// One copy of the cache (the library ping-pongs between two).
struct CacheBuf {
  void* K;       // [h_kv][cap][d] un-rotated keys
  void* V;       // [h_kv][cap][d]
  void* Kr;      // [h_kv][cap][d] keys rotated to their slot position (rope only, else NULL)
  float* S;      // [h_kv][cap] true scores
  int32_t* P;    // [h_kv][cap] original token index
  // 4-bit rows (Dims::kv_bits = 4): Kq, Vq [h_kv][cap][qstride bytes] are this copy's packed rows; K, Kr and V then
  // all point at the single bf16 staging arrays that both copies share (K = Kr = dequantized keys, rotated to
  // their slot when rope is on; V = dequantized values).
  void* Kq = nullptr;
  void* Vq = nullptr;
  int qstride = 0;
};

// tab[pos][i] = (cos, sin)(pos * theta^(-2i/d)), angles formed in double.
void launch_rope_table(float2* tab, int cap, int d, float theta, hipStream_t st);

// Weight preparation (Section 3.3).  W1t [d_R][K]: transpose of W1 with the g repeated K/V row
// blocks summed when `expand`; W2f [d_R][h_kv] float.
void launch_prep_weights(const Dims& D, int expand, const void* W1, const void* W2, void* W1t,
                         float* W2f, hipStream_t st);

// Append the chunk at slots [n_c, n_c+T) of `c`: K, V copied, Kr = K rotated to n_c+t,
// P = seen + t; qr [T][h][d] = q rotated to n_c+t (rope only; q may be NULL to skip).
// mark_unscored: also store NaN as the score of the appended units (no score will be computed).
void launch_append(const Dims& D, const void* q, const void* k, const void* v, int T, int n_c,
                   int64_t seen, const CacheBuf& c, void* qr, const float2* tab, hipStream_t st,
                   bool mark_unscored = false, const HeadLens* n_c_h = nullptr);

// 4-bit rows.  Append: quantize the chunk's k, v rows into the packed arrays of `c` at slots [n_c, n_c+T) and write
// their dequantized values (K rotated to n_c+t) into the staging arrays; P and optional NaN scores as launch_append.
// Compact: dst packed rows r = src packed rows kept[m][r], S, P likewise, staging rows r rewritten for slot r.
bool q4_head_dim(int d);
int q4_row_bytes(int d);      // d/2 code bytes + 4 bytes (scale, minimum as bf16) per group of 32 dims
int q4_row_stride(int d);     // the same, padded to a multiple of 16
void launch_append_q4(const Dims& D, const void* k, const void* v, int T, int n_c, int64_t seen, const CacheBuf& c,
                      const float2* tab, hipStream_t st, bool mark_unscored);
void launch_compact_q4(const Dims& D, const CacheBuf& src, const CacheBuf& dst, const int32_t* kept, int kept_stride,
                       int n_keep, const float2* tab, hipStream_t st);

// Attention of T queries (already rotated if rope) over slots [0, n_c+T) of Kx/V, query t seeing
// slots <= n_c+t (Eq. 1).  Reference-grade VALU kernel, any storage type.
// n_c_h (every attention launcher): per-head cache lengths, or NULL when all heads hold n_c units.
void launch_attention_simple(const Dims& D, const void* q, const void* Kx, const void* V, void* out,
                             int T, int n_c, float scale, hipStream_t st, const HeadLens* n_c_h = nullptr);
// bf16 MFMA kernel with K/V staged global -> LDS directly and the two wavefronts of every SIMD held one S block
// apart (attention_pp.hip; d = 128 or 96); false if the shape is not covered.
bool launch_attention_bf16_pp(const Dims& D, LaunchTimer tm, const void* q, const float2* tab, const void* Kx,
                              const void* V, void* out, int T, int n_c, float scale, hipStream_t st,
                              const SelectArgs* sel = nullptr, const HeadLens* n_c_h = nullptr,
                              float* split_part = nullptr, size_t split_floats = 0);
// Floats of scratch the direct-to-LDS attention kernel wants for launches that split the key range (short chunks);
// 0 when the shape never splits.  Without the buffer it does not split.
size_t attention_pp_split_floats(const Dims& D, int chunk_max);
bool attention_pp_fuses_select(const Dims& D, int n_cand);
// bf16 MFMA kernel (d in {64, 96, 128}).
void launch_attention_bf16(const Dims& D, const void* q, const void* Kx, const void* V, void* out,
                           int T, int n_c, float scale, hipStream_t st, const float2* q_rot_tab = nullptr,
                           LaunchTimer tm = LaunchTimer(), const SelectArgs* sel = nullptr,
                           const HeadLens* n_c_h = nullptr, float* split_part = nullptr, size_t split_floats = 0);
// True when launch_attention_bf16 would carry out a selection over n_cand candidates per head inside its
// own launch (pass `sel`); otherwise the caller launches launch_select itself.
bool attention_bf16_fuses_select(const Dims& D, int n_cand);
// True when launch_attention_bf16 takes un-rotated queries plus the rotary table for these
// dimensions (the kernel rotates them itself); otherwise it expects rotated queries.
bool attention_bf16_rotates_q(const Dims& D);
// True when launch_attention_bf16 attaches the LaunchTimer's events to the attention kernel's dispatch.
bool attention_bf16_attaches_timer(const Dims& D);

// Decode step (Eq. 1 with B = 1): the token q [h][d], k, v [h_kv][d] (un-rotated) attends over the n_c units of
// cache copy `c` and itself at position n_c, and is appended at slot n_c (K, V, rotated K, P = seen; with
// mark_unscored a NaN score).  n_c_h: units per KV head, n_c then being the largest.
// `part` holds h * decode_max_splits(D) * (d + 2) floats of split-K partials.
int decode_keys_per_split(const Dims& D, int n_keys);
int decode_max_splits(const Dims& D);
// pre_appended: the token already sits at slot n_c of the arrays (4-bit rows: launch_append_q4 put it there as the
// cache stores it); the launch then attends over n_c + 1 units and appends nothing.
void launch_decode_step(const Dims& D, const void* q, const void* k, const void* v, const CacheBuf& c,
                        const float2* tab, void* out, int n_c, int64_t seen, float scale, float* part, hipStream_t st,
                        bool mark_unscored, const HeadLens* n_c_h = nullptr, bool pre_appended = false);

// Retaining head: partial scores part[nb][h_kv][T] over hidden-unit blocks; returns the number of
// blocks nb through *n_parts.  `part` must hold (d_R/score_part_width) * h_kv * chunk_max floats.
int score_parts_simple(const Dims& D);
int score_parts_bf16(const Dims& D);
void launch_score_simple(const Dims& D, const void* q, const void* k, const void* v, int T,
                         const void* W1t, const float* W2f, float* part, hipStream_t st);
// Returns the number of partials it wrote (1 when it split the contraction instead, which needs `zpart`).
int launch_score_bf16(const Dims& D, const void* q, const void* k, const void* v, int T,
                      const void* W1t, const float* W2f, float* part, hipStream_t st, float* zpart = nullptr,
                      size_t zpart_floats = 0);
size_t score_bf16_split_floats(const Dims& D, int chunk_max);
// scores[m][t] = sum over nb (fixed order) -> S[m*cap + n_c + t] (if S) and out[m*T + t] (if out).
// With n_parts == 1 this is a strided copy (used for caller-supplied scores).
void launch_score_reduce(const float* part, int n_parts, int part_stride_T, int h_kv, int T, float* S,
                         int cap, int n_c, float* out, hipStream_t st, const HeadLens* n_c_h = nullptr);

// Stabilizer-masked top-k per KV head over S[m][0..L): keeps the first n_pin, the last n_stab and the
// best (n_keep - n_stab - n_pin) of the rest (score desc, index asc); kept[m][0..n_keep) ascending.
// Requires n_pin + n_stab <= min(L, n_keep).  kept2 (optional, row stride stride2) receives a copy.
void launch_select(const float* S, int cap, int h_kv, int L, int n_keep, int n_stab, int n_pin, int32_t* kept,
                   int kept_stride, int32_t* kept2, int stride2, hipStream_t st);
// The same from a filled SelectArgs (head-wise budgets: L and n_keep are the largest over the heads).
void launch_select(const SelectArgs& a, int h_kv, hipStream_t st);

// dst[m][r] = src[m][kept[m][r]] for K, V, S, P; dst.Kr[m][r] = K rotated to position r.
// keep_h: per-head row counts (n_keep then being the largest), or NULL.
void launch_compact(const Dims& D, const CacheBuf& src, const CacheBuf& dst, const int32_t* kept,
                    int kept_stride, int n_keep, const float2* tab, hipStream_t st, const HeadLens* keep_h = nullptr);

}  // namespace locret
