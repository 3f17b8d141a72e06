// Host side of the C ABI declared in include/locret.h: argument checks, workspace layout, cache
// bookkeeping (all host-known, no readbacks) and the per-chunk launch sequence.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "../../include/locret.h"
#include "kernels.h"

using namespace locret;

namespace locret {
thread_local StageTimer* tl_stage_timer = nullptr;
}

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Layout {
  size_t K[2], V[2], Kr[2], S[2], P[2];
  size_t Kq[2], Vq[2];      // 4-bit rows: the packed copies; K, V, Kr then all name the one staging pair
  size_t qr, tab, W1t, W2f, part, kept, dpart, apart, total;
  size_t apart_floats;
  size_t zpart, zpart_floats;
};

bool valid_head_dim(int d) { return d == 16 || d == 32 || d == 64 || d == 96 || d == 128; }

int validate(const locret_config* c) {
  if (!c) return LOCRET_EINVAL;
  if (c->dtype != LOCRET_F32 && c->dtype != LOCRET_BF16) return LOCRET_EINVAL;
  if (c->rope_mode != 0 && c->rope_mode != 1) return LOCRET_EINVAL;
  if (c->rh_kv_expand != 0 && c->rh_kv_expand != 1) return LOCRET_EINVAL;
  if (c->rope_mode == 1 && !(c->rope_theta > 0.f && isfinite(c->rope_theta))) return LOCRET_EINVAL;
  if (!(c->softmax_scale >= 0.f) || !isfinite(c->softmax_scale)) return LOCRET_EINVAL;
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->chunk_max < 1 || c->budget < 1 || c->d_hidden < 1)
    return LOCRET_EINVAL;
  if (c->n_q_heads % c->n_kv_heads != 0) return LOCRET_ESHAPE;
  if (!valid_head_dim(c->head_dim)) return LOCRET_ESHAPE;
  if (c->n_q_heads > 1024 || c->d_hidden > 65536) return LOCRET_ESHAPE;
  if ((int64_t)c->budget + c->chunk_max > (int64_t)1 << 28) return LOCRET_ESHAPE;
  if (c->kv_bits != 0 && c->kv_bits != 4) return LOCRET_EINVAL;
  // 4-bit rows: bf16 tensors on the matrix-core attention kernels (which rotate the queries themselves)
  if (c->kv_bits == 4 && !(c->dtype == LOCRET_BF16 && q4_head_dim(c->head_dim))) return LOCRET_ESHAPE;
  return LOCRET_OK;
}

int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  return (e && *e) ? atoi(e) : dflt;
}

// The launch switches (tests, measurements): the only place the environment is read, once per context.
Tuning tuning_from_env() {
  Tuning t;
  const char* v = getenv("LOCRET_ATTN_VARIANT");
  t.attn_regstaged = v && !strcmp(v, "regstaged");
  t.pp_split = env_int("LOCRET_PP_SPLIT", -1);
  t.pp_spread = env_int("LOCRET_PP_SPREAD", -1);
  t.score_nt = env_int("LOCRET_SCORE_NT", 0);
  t.score_split = env_int("LOCRET_SCORE_SPLIT", -1);
  const int dk = env_int("LOCRET_DEC_KEYS", 0);
  t.dec_keys = (dk >= 64 && dk <= 65536 && dk % 64 == 0) ? dk : 0;
  t.fuse_select = env_int("LOCRET_FUSE_SELECT", 1) != 0;
  return t;
}

void fill_dims(const locret_config* c, Dims* D) {
  D->tune = tuning_from_env();
  D->h = c->n_q_heads;
  D->h_kv = c->n_kv_heads;
  D->g = D->h / D->h_kv;
  D->d = c->head_dim;
  D->cap = c->budget + c->chunk_max;
  D->bf16 = c->dtype == LOCRET_BF16;
  D->rope = c->rope_mode;
  D->K = (D->h + 2 * D->h_kv) * D->d;
  D->d_R = c->d_hidden;
  D->kv_bits = c->kv_bits;
}

int max_score_parts(const Dims& D) {
  int a = score_parts_simple(D), b = score_parts_bf16(D);
  return a > b ? a : b;
}

void make_layout(const locret_config* c, const Dims& D, Layout* L) {
  const size_t es = D.bf16 ? 2 : 4;
  const size_t rows = (size_t)D.h_kv * D.cap;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up(bytes); return o; };
  if (D.kv_bits == 4) {
    const size_t kst = take(rows * D.d * es), vst = take(rows * D.d * es);      // the staging pair
    for (int i = 0; i < 2; ++i) {
      L->K[i] = L->Kr[i] = kst;
      L->V[i] = vst;
      L->Kq[i] = take(rows * q4_row_stride(D.d));
      L->Vq[i] = take(rows * q4_row_stride(D.d));
      L->S[i] = take(rows * sizeof(float));
      L->P[i] = take(rows * sizeof(int32_t));
    }
  } else {
    for (int i = 0; i < 2; ++i) {
      L->K[i] = take(rows * D.d * es);
      L->V[i] = take(rows * D.d * es);
      L->Kr[i] = D.rope ? take(rows * D.d * es) : 0;
      L->S[i] = take(rows * sizeof(float));
      L->P[i] = take(rows * sizeof(int32_t));
      L->Kq[i] = L->Vq[i] = 0;
    }
  }
  L->qr = D.rope ? take((size_t)c->chunk_max * D.h * D.d * es) : 0;
  L->tab = D.rope ? take((size_t)D.cap * (D.d / 2) * sizeof(float2)) : 0;
  L->W1t = take((size_t)D.d_R * D.K * es);
  L->W2f = take((size_t)D.d_R * D.h_kv * sizeof(float));
  L->part = take((size_t)max_score_parts(D) * D.h_kv * c->chunk_max * sizeof(float));
  L->kept = take((size_t)D.h_kv * c->budget * sizeof(int32_t));
  L->dpart = take((size_t)D.h * decode_max_splits(D) * (D.d + 2) * sizeof(float));
  L->apart_floats = attention_pp_split_floats(D, c->chunk_max);
  L->apart = take(L->apart_floats * sizeof(float));
  L->zpart_floats = score_bf16_split_floats(D, c->chunk_max);
  L->zpart = take(L->zpart_floats * sizeof(float));
  L->total = off;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// ---- scratch of the entry point that allocates nothing (locret_score_static) ------------------------------
// Device memory that lives with the code object: every GPU that loads the library holds its own copy, at its
// own address, until the process ends.  First the partial scores part[blocks][h_kv][T], then the partial
// pre-activations of launches that split the contraction.  In host code the array's name is only a handle
// for hipGetSymbolAddress; kernels and launchers get the looked-up address.
constexpr size_t STATIC_PART_FLOATS = LOCRET_STATIC_PART_FLOATS;     // 4 MiB
constexpr size_t STATIC_ZPART_FLOATS = (size_t)4 << 20;              // 16 MiB
static __device__ __align__(256) float scratch[STATIC_PART_FLOATS + STATIC_ZPART_FLOATS];

constexpr int MAX_DEVICES = 64;
float* g_scratch_ptr[MAX_DEVICES];     // per device: address of that device's copy, NULL until looked up
std::mutex g_scratch_mu;

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
int scratch_of_current_device(int* device, float** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LOCRET_EHIP; }
  *device = dev;
  *ptr = nullptr;
  if (dev < 0 || dev >= MAX_DEVICES) return LOCRET_OK;          // the static entry point then reports LOCRET_ESTATE
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return LOCRET_EHIP; }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return LOCRET_OK;
}

}  // namespace

struct locret_ctx {
  locret_config cfg;
  Dims D;
  Layout L;
  char* ws;
  int device;       // the device that was current at locret_create (the workspace's)
  float* scratch;   // that device's copy of the static scratch array, or NULL
  int cur;          // live cache copy
  int n_c;          // units per head in the live copy
  int64_t seen;     // tokens appended so far
  int have_weights;
  int n_pin;        // units at the start of the cache that no call evicts (Locret-Q's query prefix)
  // head-wise budgets: n_c is then the longest head's length
  int ragged;
  int b_h[MAX_HEAD_BUDGETS];     // budget of every KV head
  int n_c_h[MAX_HEAD_BUDGETS];   // units of every KV head in the live copy
  // the heads' lengths plus `add` in the form the launchers take, or NULL when all heads hold n_c units
  const HeadLens* lens(HeadLens* tmp, int add = 0) const {
    if (!ragged) return nullptr;
    tmp->ragged = 1;
    for (int m = 0; m < D.h_kv; ++m) tmp->v[m] = n_c_h[m] + add;
    return tmp;
  }
  int min_budget() const {
    int b = cfg.budget;
    if (ragged) for (int m = 0; m < D.h_kv; ++m) b = b_h[m] < b ? b_h[m] : b;
    return b;
  }
  float scale;
  int mfma_attn, mfma_score;
  // Selection and compaction depend on the scores only, and compaction writes the other cache copy,
  // so in the chunk step they run on a stream of the library's own beside attention (which reads
  // the live copy): forked after the retaining head, joined before the call's stream goes on.
  hipStream_t side;
  hipEvent_t ev_fork, ev_join;
  int overlap;
  std::vector<hipEvent_t> ev;   // profiling: a (begin, end) pair per stage per recorded call
  int prof_max, prof_calls;
  int prof_mode;    // 0: every stage (event packets between the kernels), 1: attention only (no extra packets),
                    // 2: every stage through the kernels' own dispatches (no extra packets)
  std::vector<uint8_t> prof_launched;   // mode 2: per recorded call, bit s set when stage s launched a kernel
  StageTimer stage_timer;
  hipEvent_t prof_event(int stage, int end) { return ev[((size_t)prof_calls * LOCRET_PROF_STAGES + stage) * 2 + end]; }
  void mark(int stage, int end, hipStream_t st) {
    if (prof_calls >= prof_max) return;
    if (prof_mode == 0) (void)hipEventRecord(ev[((size_t)prof_calls * LOCRET_PROF_STAGES + stage) * 2 + end], st);
    if (prof_mode == 2) {
      // the launches between mark(stage, 0) and mark(stage, 1) carry the stage's events themselves
      if (end == 0) {
        stage_timer.start = prof_event(stage, 0);
        stage_timer.stop = prof_event(stage, 1);
        stage_timer.launches = 0;
        tl_stage_timer = &stage_timer;
      } else {
        if (stage_timer.launches > 0) prof_launched[prof_calls] |= (uint8_t)(1u << stage);
        tl_stage_timer = nullptr;
      }
    }
  }
  CacheBuf buf(int i) const {
    CacheBuf b;
    b.K = ws + L.K[i];
    b.V = ws + L.V[i];
    b.Kr = (D.rope || D.kv_bits) ? ws + L.Kr[i] : nullptr;
    b.S = (float*)(ws + L.S[i]);
    b.P = (int32_t*)(ws + L.P[i]);
    if (D.kv_bits) {
      b.Kq = ws + L.Kq[i];
      b.Vq = ws + L.Vq[i];
      b.qstride = q4_row_stride(D.d);
    }
    return b;
  }
};

extern "C" {

size_t locret_workspace_bytes(const locret_config* cfg) {
  if (validate(cfg) != LOCRET_OK) return 0;
  Dims D;
  fill_dims(cfg, &D);
  Layout L;
  make_layout(cfg, D, &L);
  return L.total;
}

int locret_create(const locret_config* cfg, void* ws, size_t bytes, locret_ctx** out) {
  if (!out) return LOCRET_EINVAL;
  int rc = validate(cfg);
  if (rc != LOCRET_OK) return rc;
  if (!ws) return LOCRET_EINVAL;
  if (((uintptr_t)ws & (ALIGN - 1)) != 0) return LOCRET_EALIGN;
  locret_ctx* c = new (std::nothrow) locret_ctx();
  if (!c) return LOCRET_ENOMEM;
  c->cur = 0; c->n_c = 0; c->seen = 0; c->have_weights = 0; c->prof_max = 0; c->prof_calls = 0;
  c->side = nullptr; c->ev_fork = nullptr; c->ev_join = nullptr; c->overlap = 0; c->n_pin = 0; c->prof_mode = 0;
  c->ragged = 0;
  c->cfg = *cfg;
  fill_dims(cfg, &c->D);
  make_layout(cfg, c->D, &c->L);
  if (bytes < c->L.total) { delete c; return LOCRET_ENOMEM; }
  c->ws = (char*)ws;
  c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
  if (scratch_of_current_device(&c->device, &c->scratch) != LOCRET_OK) { delete c; return LOCRET_EHIP; }
  const char* force = getenv("LOCRET_FORCE_SIMPLE");
  const bool simple = force && force[0] == '1';
  const int d = cfg->head_dim;
  c->mfma_attn = !simple && c->D.bf16 && (d == 64 || d == 96 || d == 128);
  c->mfma_score = !simple && c->D.bf16 && score_parts_bf16(c->D) > 0;
  if (c->D.kv_bits && !c->mfma_attn) { delete c; return LOCRET_ESHAPE; }   // 4-bit rows: matrix-core attention only
  if (c->D.rope) {
    launch_rope_table((float2*)(c->ws + c->L.tab), c->D.cap, c->D.d, cfg->rope_theta, 0);
    if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) { delete c; return LOCRET_EHIP; }
  } else if (hipDeviceSynchronize() != hipSuccess) {   // also proves a device is usable
    (void)hipGetLastError();
    delete c;
    return LOCRET_EHIP;
  }
  // LOCRET_OVERLAP=1 (read here, per context): run selection and compaction beside attention.
  // Off by default: measured on config 3 it gains 1.6 % per step (the selection's 1024-thread
  // workgroups do not fit on a CU next to an attention workgroup, so they start only when the first
  // attention workgroups retire) and it blurs the per-stage timings.
  const char* ov = getenv("LOCRET_OVERLAP");
  c->overlap = ov && ov[0] == '1';
  c->side = nullptr; c->ev_fork = nullptr; c->ev_join = nullptr;
  if (c->overlap) {
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      locret_destroy(c);
      return LOCRET_EHIP;
    }
  }
  *out = c;
  return LOCRET_OK;
}

int locret_set_weights(locret_ctx* c, const void* W1, const void* W2, void* stream) {
  if (!c || !W1 || !W2) return LOCRET_EINVAL;
  if (misaligned(W1) || misaligned(W2)) return LOCRET_EALIGN;
  launch_prep_weights(c->D, c->cfg.rh_kv_expand, W1, W2, c->ws + c->L.W1t, (float*)(c->ws + c->L.W2f),
                      (hipStream_t)stream);
  if (hipGetLastError() != hipSuccess) return LOCRET_EHIP;
  c->have_weights = 1;
  return LOCRET_OK;
}

int locret_set_pinned_prefix(locret_ctx* c, int32_t n_pin) {
  if (!c || n_pin < 0 || n_pin > c->cfg.budget) return LOCRET_EINVAL;
  c->n_pin = n_pin;
  return LOCRET_OK;
}

int locret_set_head_budgets(locret_ctx* c, const int32_t* budgets) {
  if (!c) return LOCRET_EINVAL;
  if (c->n_c != 0) return LOCRET_ESTATE;
  if (!budgets) { c->ragged = 0; return LOCRET_OK; }
  if (c->D.h_kv > MAX_HEAD_BUDGETS || c->D.kv_bits) return LOCRET_ESHAPE;
  for (int m = 0; m < c->D.h_kv; ++m)
    if (budgets[m] < 1 || budgets[m] > c->cfg.budget) return LOCRET_EINVAL;
  for (int m = 0; m < c->D.h_kv; ++m) { c->b_h[m] = budgets[m]; c->n_c_h[m] = 0; }
  c->ragged = 1;
  return LOCRET_OK;
}

int locret_reset(locret_ctx* c) {
  if (!c) return LOCRET_EINVAL;
  c->n_c = 0;
  c->seen = 0;
  for (int m = 0; m < MAX_HEAD_BUDGETS; ++m) c->n_c_h[m] = 0;
  return LOCRET_OK;
}

// reduce = false: only the partial scores are formed (ws + L.part, *n_parts of them); the caller sums them
// part / zpart: where the partial scores and (split launches) partial pre-activations go; NULL part = the
// workspace's buffers
static void run_score(locret_ctx* c, const void* q, const void* k, const void* v, int T, float* S_dst, int n_c,
                      float* out, hipStream_t st, bool reduce = true, int* n_parts = nullptr, float* part = nullptr,
                      float* zpart = nullptr, size_t zpart_floats = 0) {
  HeadLens hl_tmp;
  if (!part) {
    part = (float*)(c->ws + c->L.part);
    zpart = c->L.zpart_floats ? (float*)(c->ws + c->L.zpart) : nullptr;
    zpart_floats = c->L.zpart_floats;
  }
  int parts;
  if (c->mfma_score) {
    parts = launch_score_bf16(c->D, q, k, v, T, c->ws + c->L.W1t, (const float*)(c->ws + c->L.W2f), part, st,
                              zpart_floats ? zpart : nullptr, zpart_floats);
  } else {
    launch_score_simple(c->D, q, k, v, T, c->ws + c->L.W1t, (const float*)(c->ws + c->L.W2f), part, st);
    parts = score_parts_simple(c->D);
  }
  if (n_parts) *n_parts = parts;
  if (reduce) launch_score_reduce(part, parts, T, c->D.h_kv, T, S_dst, c->D.cap, n_c, out, st, c->lens(&hl_tmp));
}

// the selection over the live copy's rows [0, L)
static SelectArgs select_args(locret_ctx* c, int L, int n_stab, int32_t* kept_idx_out) {
  const int b = c->cfg.budget;
  const int n_keep = L < b ? L : b;
  const int ns = n_stab < L ? n_stab : L;
  const int npin = c->n_pin < L - ns ? c->n_pin : L - ns;     // the prefix covers what the stabilizers leave
  CacheBuf A = c->buf(c->cur);
  SelectArgs a = {A.S, c->D.cap, L, n_keep, ns, npin, (int32_t*)(c->ws + c->L.kept), b, kept_idx_out, b,
                  nullptr, 0, 0, 0, 0, nullptr, nullptr};
  a.L_h.ragged = a.keep_h.ragged = c->ragged;
  if (c->ragged) {
    // L is the longest head's length (it sizes the launch); every head clamps n_stab and n_pin to its own
    a.n_keep = 0;
    for (int m = 0; m < c->D.h_kv; ++m) {
      const int Lm = c->n_c_h[m] + (L - c->n_c);
      a.L_h.v[m] = Lm;
      a.keep_h.v[m] = Lm < c->b_h[m] ? Lm : c->b_h[m];
      a.n_keep = a.keep_h.v[m] > a.n_keep ? a.keep_h.v[m] : a.n_keep;
    }
  }
  return a;
}

// select + compact on the live copy, whose rows [0, L) are filled; updates the host bookkeeping.
// select_done: the selection has already been launched (inside the attention launch).
static void run_evict(locret_ctx* c, int L, int n_stab, int32_t* kept_idx_out, hipStream_t st, bool select_done = false) {
  const int b = c->cfg.budget;
  const SelectArgs a = select_args(c, L, n_stab, kept_idx_out);
  CacheBuf A = c->buf(c->cur);
  c->mark(3, 0, st);
  if (!select_done) launch_select(a, c->D.h_kv, st);
  c->mark(3, 1, st);
  c->mark(4, 0, st);
  // the other copy becomes the live one as soon as one head is over its budget; the heads that are not
  // are then copied as they are (their kept lists are 0, 1, 2, ...)
  bool over = L > b;
  if (c->ragged) {
    over = false;
    for (int m = 0; m < c->D.h_kv; ++m) over = over || a.L_h.v[m] > c->b_h[m];
  }
  if (over) {
    CacheBuf B = c->buf(c->cur ^ 1);
    const float2* tab = c->D.rope ? (const float2*)(c->ws + c->L.tab) : nullptr;
    if (c->D.kv_bits) launch_compact_q4(c->D, A, B, a.kept, b, a.n_keep, tab, st);
    else launch_compact(c->D, A, B, a.kept, b, a.n_keep, tab, st, c->ragged ? &a.keep_h : nullptr);
    c->cur ^= 1;
  }
  c->mark(4, 1, st);
  c->n_c = a.n_keep;
  if (c->ragged) for (int m = 0; m < c->D.h_kv; ++m) c->n_c_h[m] = a.keep_h.v[m];
}

// the cache grew by T units in every head and nothing was evicted
static void grow(locret_ctx* c, int T) {
  c->n_c += T;
  if (c->ragged) for (int m = 0; m < c->D.h_kv; ++m) c->n_c_h[m] += T;
}

int locret_prefill_chunk(locret_ctx* c, const void* q, const void* k, const void* v, int32_t T, int32_t n_stab,
                         int32_t evict, const float* scores_in, void* attn_out, float* scores_out,
                         int32_t* kept_idx_out, void* stream) {
  if (!c || !q || !k || !v || !attn_out) return LOCRET_EINVAL;
  if (n_stab < 0 || n_stab > c->cfg.budget) return LOCRET_EINVAL;
  if (evict && n_stab + c->n_pin > c->min_budget()) return LOCRET_EINVAL;
  if (T < 1 || T > c->cfg.chunk_max) return LOCRET_ESHAPE;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(attn_out) || misaligned(scores_in) ||
      misaligned(scores_out) || misaligned(kept_idx_out))
    return LOCRET_EALIGN;
  if (!c->have_weights) return LOCRET_ESTATE;
  if (c->n_c + T > c->D.cap) return LOCRET_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  const Dims& D = c->D;
  CacheBuf A = c->buf(c->cur);
  const float2* tab = D.rope ? (const float2*)(c->ws + c->L.tab) : nullptr;
  void* qr = D.rope ? c->ws + c->L.qr : nullptr;

  // the matrix-core attention kernels rotate the queries themselves: no rotated copy is written or read
  const bool fused_q = c->mfma_attn && attention_bf16_rotates_q(D);
  HeadLens hl_tmp;
  const HeadLens* hl = c->lens(&hl_tmp);      // per-head cache lengths before this chunk, or NULL
  c->mark(0, 0, st);
  if (D.kv_bits) launch_append_q4(D, k, v, T, c->n_c, c->seen, A, tab, st, false);
  else launch_append(D, fused_q ? nullptr : q, k, v, T, c->n_c, c->seen, A, qr, tab, st, false, hl);
  c->mark(0, 1, st);
  const void* qx = (D.rope && !fused_q) ? qr : q;
  const void* Kx = D.rope ? A.Kr : A.K;
  const int n_c = c->n_c;
  const int L = n_c + T;
  float* split_part = c->L.apart_floats ? (float*)(c->ws + c->L.apart) : nullptr;
  auto attention = [&](const SelectArgs* sel) {
    // when profiling, the matrix-core kernels are timed through their own dispatch
    const bool prof = c->prof_calls < c->prof_max;
    if (c->mfma_attn && prof && attention_bf16_attaches_timer(D)) {
      LaunchTimer tm;
      tm.start = c->prof_event(1, 0);
      tm.stop = c->prof_event(1, 1);
      launch_attention_bf16(D, qx, Kx, A.V, attn_out, T, n_c, c->scale, st, fused_q ? tab : nullptr, tm, sel, hl,
                            split_part, c->L.apart_floats);
      if (c->prof_mode == 2) c->prof_launched[c->prof_calls] |= 1u << 1;
      return;
    }
    c->mark(1, 0, st);
    if (c->mfma_attn) launch_attention_bf16(D, qx, Kx, A.V, attn_out, T, n_c, c->scale, st, fused_q ? tab : nullptr, LaunchTimer(), sel, hl,
                                            split_part, c->L.apart_floats);
    else launch_attention_simple(D, qx, Kx, A.V, attn_out, T, n_c, c->scale, st, hl);
    c->mark(1, 1, st);
  };
  auto scores = [&](SelectArgs* fused) {
    c->mark(2, 0, st);
    if (fused && !scores_in) {
      // the selection workgroups of the attention launch sum the partial scores themselves
      int parts = 0;
      run_score(c, q, k, v, T, nullptr, n_c, nullptr, st, /*reduce=*/false, &parts);
      fused->part = (const float*)(c->ws + c->L.part);
      fused->n_parts = parts;
      fused->part_T = T;
      fused->h_kv = D.h_kv;
      fused->red_T = T;
      fused->S_w = A.S;
      fused->red_out = scores_out;
    } else {
      run_score(c, q, k, v, T, scores_in ? nullptr : A.S, n_c, scores_out, st);
      if (scores_in) launch_score_reduce(scores_in, 1, T, D.h_kv, T, A.S, D.cap, n_c, nullptr, st, hl);
    }
    c->mark(2, 1, st);
  };
  bool ok = true;
  // The selection depends on the scores only.  Where the attention launch can carry it (direct-to-LDS kernel, head_dim 128 or 96,
  // few enough candidates for its register-resident form) the retaining head runs first and the selection
  // rides in the first workgroups of the attention launch (Tuning::fuse_select = 0 keeps the separate launch).
  bool fuse_select = false;
  SelectArgs sa{};
  if (evict && !c->overlap && c->mfma_attn) {
    sa = select_args(c, L, n_stab, kept_idx_out);
    fuse_select = attention_bf16_fuses_select(D, sa.L - sa.n_stab - sa.n_pin);
  }
  if (evict && c->overlap) {
    scores(nullptr);
    ok = ok && hipEventRecord(c->ev_fork, st) == hipSuccess;
    ok = ok && hipStreamWaitEvent(c->side, c->ev_fork, 0) == hipSuccess;
    run_evict(c, L, n_stab, kept_idx_out, c->side);
    ok = ok && hipEventRecord(c->ev_join, c->side) == hipSuccess;
    attention(nullptr);
    ok = ok && hipStreamWaitEvent(st, c->ev_join, 0) == hipSuccess;
  } else if (fuse_select) {
    scores(&sa);
    attention(&sa);
    run_evict(c, L, n_stab, kept_idx_out, st, /*select_done=*/true);
  } else {
    attention(nullptr);
    scores(nullptr);
    if (evict) run_evict(c, L, n_stab, kept_idx_out, st);
    else {
      grow(c, T);
      c->mark(3, 0, st); c->mark(3, 1, st); c->mark(4, 0, st); c->mark(4, 1, st);
    }
  }
  if (c->prof_calls < c->prof_max) c->prof_calls++;
  c->seen += T;
  return (hipGetLastError() == hipSuccess && ok) ? LOCRET_OK : LOCRET_EHIP;
}

int locret_decode_step(locret_ctx* c, const void* q, const void* k, const void* v, int32_t with_score,
                       void* attn_out, float* scores_out, void* stream) {
  if (!c || !q || !k || !v || !attn_out) return LOCRET_EINVAL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(attn_out)) return LOCRET_EALIGN;
  if (with_score && !c->have_weights) return LOCRET_ESTATE;
  if (c->n_c + 1 > c->D.cap) return LOCRET_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  const Dims& D = c->D;
  CacheBuf A = c->buf(c->cur);
  const float2* tab = D.rope ? (const float2*)(c->ws + c->L.tab) : nullptr;
  HeadLens hl_tmp;
  if (with_score) run_score(c, q, k, v, 1, A.S, c->n_c, scores_out, st);
  // 4-bit rows: the token enters the cache first (packed row + staging), then attention reads it like any unit
  if (D.kv_bits) launch_append_q4(D, k, v, 1, c->n_c, c->seen, A, tab, st, /*mark_unscored=*/!with_score);
  launch_decode_step(D, q, k, v, A, tab, attn_out, c->n_c, c->seen, c->scale, (float*)(c->ws + c->L.dpart), st,
                     /*mark_unscored=*/!with_score, c->lens(&hl_tmp), /*pre_appended=*/D.kv_bits != 0);
  grow(c, 1);
  c->seen += 1;
  return hipGetLastError() == hipSuccess ? LOCRET_OK : LOCRET_EHIP;
}

int locret_score(locret_ctx* c, const void* q, const void* k, const void* v, int32_t T, float* scores,
                 void* stream) {
  if (!c || !q || !k || !v || !scores) return LOCRET_EINVAL;
  if (T < 1 || T > c->cfg.chunk_max) return LOCRET_ESHAPE;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(scores)) return LOCRET_EALIGN;
  if (!c->have_weights) return LOCRET_ESTATE;
  run_score(c, q, k, v, T, nullptr, 0, scores, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? LOCRET_OK : LOCRET_EHIP;
}

int locret_score_static(locret_ctx* c, const void* q, const void* k, const void* v, int32_t T, float* scores,
                        void* stream) {
  if (!c || !q || !k || !v || !scores) return LOCRET_EINVAL;
  if (T < 1 || T > c->cfg.chunk_max) return LOCRET_ESHAPE;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(scores)) return LOCRET_EALIGN;
  if (!c->have_weights || !c->scratch) return LOCRET_ESTATE;
  const int parts = c->mfma_score ? score_parts_bf16(c->D) : score_parts_simple(c->D);     // of the kernel that will run
  if ((size_t)parts * c->D.h_kv * (size_t)T > STATIC_PART_FLOATS) return LOCRET_ELIMIT;
  // the launcher splits the contraction exactly as locret_score does while the slices fit the static region
  const size_t zf = c->L.zpart_floats < STATIC_ZPART_FLOATS ? c->L.zpart_floats : STATIC_ZPART_FLOATS;
  run_score(c, q, k, v, T, nullptr, 0, scores, (hipStream_t)stream, true, nullptr, c->scratch,
            c->scratch + STATIC_PART_FLOATS, zf);
  return hipGetLastError() == hipSuccess ? LOCRET_OK : LOCRET_EHIP;
}

int locret_evict_compact(locret_ctx* c, const float* chunk_scores, const void* k, const void* v, int32_t T,
                         int32_t n_stab, int32_t* kept_idx_out, void* stream) {
  if (!c || !chunk_scores || !k || !v) return LOCRET_EINVAL;
  if (n_stab < 0 || n_stab + c->n_pin > c->min_budget()) return LOCRET_EINVAL;
  if (T < 1 || T > c->cfg.chunk_max) return LOCRET_ESHAPE;
  if (misaligned(chunk_scores) || misaligned(k) || misaligned(v) || misaligned(kept_idx_out)) return LOCRET_EALIGN;
  if (c->n_c + T > c->D.cap) return LOCRET_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  const Dims& D = c->D;
  CacheBuf A = c->buf(c->cur);
  const float2* tab = D.rope ? (const float2*)(c->ws + c->L.tab) : nullptr;
  HeadLens hl_tmp;
  const HeadLens* hl = c->lens(&hl_tmp);
  if (D.kv_bits) launch_append_q4(D, k, v, T, c->n_c, c->seen, A, tab, st, false);
  else launch_append(D, nullptr, k, v, T, c->n_c, c->seen, A, nullptr, tab, st, false, hl);
  launch_score_reduce(chunk_scores, 1, T, D.h_kv, T, A.S, D.cap, c->n_c, nullptr, st, hl);
  run_evict(c, c->n_c + T, n_stab, kept_idx_out, st);
  c->seen += T;
  return hipGetLastError() == hipSuccess ? LOCRET_OK : LOCRET_EHIP;
}

int32_t locret_cache_len(const locret_ctx* c) { return c ? c->n_c : LOCRET_EINVAL; }
int locret_cache_lens(const locret_ctx* c, int32_t* lens) {
  if (!c || !lens) return LOCRET_EINVAL;
  for (int m = 0; m < c->D.h_kv; ++m) lens[m] = c->ragged ? c->n_c_h[m] : c->n_c;
  return LOCRET_OK;
}
int64_t locret_tokens_seen(const locret_ctx* c) { return c ? c->seen : (int64_t)LOCRET_EINVAL; }

int locret_cache_view(const locret_ctx* c, const void** K, const void** V, const float** score,
                      const int32_t** orig_pos, int32_t* len, int32_t* row_stride) {
  if (!c) return LOCRET_EINVAL;
  CacheBuf A = c->buf(c->cur);
  if (K) *K = c->D.kv_bits ? nullptr : A.K;       // 4-bit rows: no un-rotated bf16 keys exist (locret_cache_view_q4)
  if (V) *V = A.V;
  if (score) *score = A.S;
  if (orig_pos) *orig_pos = A.P;
  if (len) *len = c->n_c;
  if (row_stride) *row_stride = c->D.cap;
  return LOCRET_OK;
}

int locret_cache_view_q4(const locret_ctx* c, const void** Kq, const void** Vq, int32_t* len, int32_t* row_stride,
                         int32_t* row_bytes, int32_t* row_stride_bytes) {
  if (!c) return LOCRET_EINVAL;
  if (!c->D.kv_bits) return LOCRET_ESTATE;
  CacheBuf A = c->buf(c->cur);
  if (Kq) *Kq = A.Kq;
  if (Vq) *Vq = A.Vq;
  if (len) *len = c->n_c;
  if (row_stride) *row_stride = c->D.cap;
  if (row_bytes) *row_bytes = q4_row_bytes(c->D.d);
  if (row_stride_bytes) *row_stride_bytes = A.qstride;
  return LOCRET_OK;
}

static void free_events(locret_ctx* c) {
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  c->ev.clear();
  c->prof_max = c->prof_calls = 0;
}

int locret_profile_enable(locret_ctx* c, int32_t max_calls) {
  if (!c || max_calls < 0 || max_calls > 65536) return LOCRET_EINVAL;
  free_events(c);
  if (max_calls == 0) return LOCRET_OK;
  const size_t n = (size_t)max_calls * LOCRET_PROF_STAGES * 2;
  c->ev.reserve(n);
  for (size_t i = 0; i < n; ++i) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) { free_events(c); return LOCRET_EHIP; }
    c->ev.push_back(e);
  }
  c->prof_max = max_calls;
  c->prof_launched.assign((size_t)max_calls, 0);
  return LOCRET_OK;
}

int locret_profile_mode(locret_ctx* c, int32_t mode) {
  if (!c || mode < 0 || mode > 2) return LOCRET_EINVAL;
  if (c->prof_calls != 0) return LOCRET_ESTATE;       // read or re-arm first
  c->prof_mode = mode;
  return LOCRET_OK;
}

int locret_profile_read(locret_ctx* c, double* stage_ms, int32_t* n_calls) {
  if (!c || !stage_ms || !n_calls) return LOCRET_EINVAL;
  for (int s = 0; s < LOCRET_PROF_STAGES; ++s) stage_ms[s] = 0.0;
  *n_calls = c->prof_calls;
  const bool attn_only = c->prof_mode == 1;
  if (attn_only && !(c->mfma_attn && attention_bf16_attaches_timer(c->D))) {   // nothing was time-stamped
    c->prof_calls = 0;
    *n_calls = 0;
    return LOCRET_OK;
  }
  for (int i = 0; i < c->prof_calls; ++i) {
    hipEvent_t* e = &c->ev[(size_t)i * LOCRET_PROF_STAGES * 2];
    for (int s = 0; s < LOCRET_PROF_STAGES; ++s) {
      if (attn_only && s != 1) continue;
      if (c->prof_mode == 2 && !(c->prof_launched[i] & (1u << s))) continue;     // the stage launched nothing
      float ms = 0.f;
      if (hipEventSynchronize(e[2 * s + 1]) != hipSuccess) return LOCRET_EHIP;
      if (hipEventElapsedTime(&ms, e[2 * s], e[2 * s + 1]) != hipSuccess) return LOCRET_EHIP;
      stage_ms[s] += ms;
    }
  }
  c->prof_calls = 0;
  std::fill(c->prof_launched.begin(), c->prof_launched.end(), (uint8_t)0);
  return LOCRET_OK;
}

void locret_destroy(locret_ctx* c) {
  if (!c) return;
  free_events(c);
  if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  delete c;
}

const char* locret_strerror(int code) {
  switch (code) {
    case LOCRET_OK: return "ok";
    case LOCRET_EINVAL: return "invalid argument (null pointer or value outside its domain)";
    case LOCRET_ESHAPE: return "unsupported shape (head layout, head_dim, or T outside 1..chunk_max)";
    case LOCRET_EALIGN: return "device pointer not 16-byte aligned (workspace: 256-byte)";
    case LOCRET_ESTATE: return "call not valid in this state (weights not set, or cache capacity exceeded)";
    case LOCRET_EHIP: return "HIP runtime error";
    case LOCRET_ENOMEM: return "workspace too small or host allocation failed";
    case LOCRET_ELIMIT: return "size beyond the static scratch of the entry point that allocates nothing";
    default: return "unknown error code";
  }
}

}  // extern "C"
