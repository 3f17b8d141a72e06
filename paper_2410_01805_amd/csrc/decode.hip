// Decode step: attention of ONE new token over the retained cache (Eq. 1 with B = 1; the generate
// step that closes Algorithm 1).  The work is a single pass over K and V of every KV head, so the
// kernel is built for HBM bandwidth: no matrix cores, no LDS staging.
//
// Split-K over the key axis: workgroup (split, m) owns DEC_KEYS keys of KV head m and serves the
// query heads of its group (G at a time).  A key row is spread over LPR lanes (16 bytes per lane,
// padded to a power of two), so one load instruction of a wavefront fetches 64 / LPRP whole rows,
// contiguous in memory.  Logits: with bf16 storage and head dims that are multiples of 32 the wavefront's 16
// (or 32) rows of an iteration form one S^T = K Q^T product on the matrix cores (v_mfma_f32_16x16x32_bf16:
// rows = keys, fetched from memory straight into the A-operand layout; columns = the G query heads, padded to
// 16), and the logits reach the lanes that own the rows through 256 bytes of LDS per wavefront; the matrix cores
// idle most of the time here, but the G dot products per row with their butterflies over the row's lanes were
// more than half of the vector instructions and kept the kernel from overlapping them with its loads.  Other
// types: each lane keeps the query values of its own dims for G heads and a logit is G short dot products plus a
// butterfly over the lanes of the row.  Either way the lanes of a row then share the probability and accumulate
// p * v for their dims.  Online softmax with a lazily raised max as in
// the prefill kernels, one decision per UN rows.  The (max, sum, vector) triples of the 16 or 32
// row slots of a workgroup are merged through LDS, those of the splits by decode_merge_kernel.
//
// The step is two launches.  The split kernel goes over the units already in the cache and rotates the
// (un-rotated) query itself; one more workgroup per KV head takes the new token: one more partial (logit from
// the rotated query and key, value row, sum 1) and the append to the cache (K, V, the rotated-key shadow, the
// original position, and a NaN score when the caller does not score generated tokens).  The merge kernel
// combines the partials.  A separate append launch cost 15 % of the step.
#include <stdlib.h>

#include <type_traits>

#include "attn_common.h"
#include "kernels.h"

namespace locret {

constexpr int DEC_THREADS = 256;
constexpr int DEC_UN = 4;               // rows per lane group between max decisions
constexpr float DEC_RESCALE_LOG2 = 8.f;

template <int X> struct Pow2Ceil { static constexpr int value = X <= 1 ? 1 : 2 * Pow2Ceil<(X + 1) / 2>::value; };
template <> struct Pow2Ceil<1> { static constexpr int value = 1; };

// The new token of a decode step and where it goes (all device pointers; q, k, v un-rotated).
struct DecodeToken {
  const void* q;          // [h][d]
  const void* k;          // [h_kv][d]
  const void* v;          // [h_kv][d]
  const float2* tab;      // rotary table, or NULL
  void* K;                // cache arrays of the live copy
  void* V;
  void* Kr;
  float* S;
  int32_t* P;
  int g, cap, n_c, seen, mark_unscored;
  int pre;                // 1: the token is already at slot n_c; attend over n_c + 1 units, no token workgroup
  float c_log2;
  HeadLens n_c_h;         // units per head before the token (ragged), else n_c
};

template <typename T, int D, int G>
__global__ __launch_bounds__(DEC_THREADS) void decode_attn_kernel(const T* __restrict__ Kx, int g0, int keys_per_wg,
                                                                  float* __restrict__ part, DecodeToken tk) {
  // n_splits partials per query head: gridDim.x - 1 splits over the cached units, then the new token's, which the
  // last workgroup of a head forms (it has no units of its own, so it is done long before the others)
  const T* __restrict__ q = (const T*)tk.q;
  const T* __restrict__ V = (const T*)tk.V;
  const float2* __restrict__ tab = tk.tab;
  const int g = tk.g, cap = tk.cap, n_splits = (int)gridDim.x;
  const float c_log2 = tk.c_log2;
  constexpr int VEC = Vec16<T>::N;
  constexpr int LPR = D / VEC;                       // lanes that hold data of one row
  constexpr int LPRP = Pow2Ceil<LPR>::value;         // lanes reserved per row
  constexpr int KPW = 64 / LPRP;                     // rows per wavefront per load
  constexpr int NSETS = (DEC_THREADS / 64) * KPW;    // row slots per workgroup
  constexpr int PW = D + 2;                          // floats per partial: vector, max, sum
  typedef Vec16<T> V16;
  typedef decltype(V16().raw) raw_t;
  __shared__ float sets[NSETS * G * PW];
  // logits on the matrix cores (see the file header)
  constexpr bool MM = std::is_same<T, bf16_t>::value && D % 32 == 0 && G <= 16 && (DEC_UN * KPW) % 16 == 0;
  constexpr int WROWS = DEC_UN * KPW;                // rows of a wavefront per iteration
  constexpr int NSB = MM ? WROWS / 16 : 1;           // 16-row blocks among them
  constexpr int NKS = MM ? D / 32 : 1;               // contraction steps
  __shared__ float slog[MM ? (DEC_THREADS / 64) * WROWS * G : 1];

  const int split = blockIdx.x, m = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPRP, grp = lane / LPRP;
  const bool act = sub < LPR;
  // head-wise budgets: a head shorter than the longest leaves its last splits empty (k1 <= k0: no row is
  // read, the partial carries max -inf and sum 0, which the merge weighs with 0)
  const int n_keys = head_len(tk.n_c_h, m, tk.n_c);   // units of this head in the cache = the new token's slot and position
  const int k0 = split * keys_per_wg;
  const int k1 = min(n_keys + tk.pre, k0 + keys_per_wg);
  const T* Kb = Kx + (int64_t)m * cap * D;
  const T* Vb = V + (int64_t)m * cap * D;
  const int off = (act ? sub : 0) * VEC;

  // `tab` non-null: q is un-rotated and takes position n_keys (the slot the token is appended at).  One thread
  // per 16-byte chunk of the G query rows rotates its dims with the partner dims (+- D/2), rounds to the storage
  // type as the rotated query of a chunk is, and leaves the row in LDS for the whole workgroup: every workgroup
  // of the launch reads the same few lines of q and of the table, and those requests queue on one L2 channel
  // (with every lane rotating for itself the kernel took 26 us instead of 20).
  float qv[G][VEC];
  __shared__ float qs[G * D];
  if (tab != nullptr) {
    constexpr int CPR = D / VEC;                       // chunks per row
    if (tid < G * CPR) {
      const int u = tid / CPR, offc = (tid % CPR) * VEC;
      const int j = m * g + min(g0 + u, g - 1);
      const bool low = offc < D / 2;
      V16 x, y;
      x.raw = *(const raw_t*)(q + (int64_t)j * D + offc);
      y.raw = *(const raw_t*)(q + (int64_t)j * D + (low ? offc + D / 2 : offc - D / 2));
      const float2* tr = tab + (int64_t)n_keys * (D / 2) + (low ? offc : offc - D / 2);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float2 cs = tr[e];
        V16 r;
        r.set(0, low ? x.get(e) * cs.x - y.get(e) * cs.y : x.get(e) * cs.x + y.get(e) * cs.y);
        qs[u * D + offc + e] = r.get(0) * c_log2;      // logits in log2 units
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < G; ++u)
#pragma unroll
      for (int e = 0; e < VEC; ++e) qv[u][e] = act ? qs[u * D + off + e] : 0.f;
  } else {
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int j = m * g + min(g0 + u, g - 1);        // spare heads repeat the last one (not written)
      V16 x;
      x.raw = *(const raw_t*)(q + (int64_t)j * D + off);
#pragma unroll
      for (int e = 0; e < VEC; ++e) qv[u][e] = act ? x.get(e) * c_log2 : 0.f;   // logits in log2 units
    }
    if (MM) {                                          // the matrix-core path takes the query from LDS
      if (act && grp == 0 && wave == 0)
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
          for (int e = 0; e < VEC; ++e) qs[u * D + off + e] = qv[u][e];
      __syncthreads();
    }
  }
  // B operand of S^T = K Q^T: lane (head n = lane % 16, k group lane / 16) holds q[n][32 ks + 8 (lane / 16) .. + 8],
  // scaled, rounded to bf16 (as the chunk kernels round their pre-scaled queries); heads past G are zero
  bf16x8 qb[NKS];
  if (MM) {
    const int n = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = n < G ? qs[n * D + ks * 32 + kg * 8 + e] : 0.f;
      const uint4 pk = make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
      qb[ks] = __builtin_bit_cast(bf16x8, pk);
    }
  }
  float o[G][VEC], mrun[G], lrun[G];
#pragma unroll
  for (int u = 0; u < G; ++u) {
    mrun[u] = -INFINITY;
    lrun[u] = 0.f;
#pragma unroll
    for (int e = 0; e < VEC; ++e) o[u][e] = 0.f;
  }

  constexpr int BLK = (DEC_THREADS / 64) * DEC_UN * KPW;   // rows per workgroup iteration
  for (int kb = k0; kb < k1; kb += BLK) {
    V16 kf[MM ? 1 : DEC_UN], vf[DEC_UN];
    bool valid[DEC_UN];
    bf16x8 ka[NSB][NKS];
    if (MM) {
      // A operand: lane (row lane % 16 of the 16-row block, k group lane / 16) fetches 16 bytes of that key's row
      const bf16_t* Kh = (const bf16_t*)Kb;
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
        const int key = kb + wave * WROWS + sb * 16 + (lane & 15);
        const bf16_t* kr = Kh + (int64_t)(key < k1 ? key : k0) * D + (lane >> 4) * 8;    // spare rows re-read the first row
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) ka[sb][ks] = *(const bf16x8*)(kr + ks * 32);
      }
    }
#pragma unroll
    for (int i = 0; i < DEC_UN; ++i) {
      const int key = kb + (wave * DEC_UN + i) * KPW + grp;
      valid[i] = key < k1;
      const int64_t row = (int64_t)(valid[i] ? key : k0) * D + off;   // spare slots re-read the first row
      if (!MM) kf[i].raw = *(const raw_t*)(Kb + row);
      vf[i].raw = *(const raw_t*)(Vb + row);
    }
    float s[DEC_UN][G];
    if (MM) {
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      float* sl = slog + wave * (WROWS * G);
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[sb][ks], qb[ks], acc, 0, 0, 0);
        // the lane holds rows 4 (lane / 16) + r of the block for head lane % 16
        if ((lane & 15) < G)
#pragma unroll
          for (int r = 0; r < 4; ++r) sl[(sb * 16 + 4 * (lane >> 4) + r) * G + (lane & 15)] = acc[r];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int i = 0; i < DEC_UN; ++i)
#pragma unroll
        for (int u = 0; u < G; ++u) s[i][u] = valid[i] ? sl[(i * KPW + grp) * G + u] : -INFINITY;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();                  // the next iteration rewrites the tile
    } else {
#pragma unroll
      for (int i = 0; i < DEC_UN; ++i)
#pragma unroll
        for (int u = 0; u < G; ++u) {
          float a = 0.f;
#pragma unroll
          for (int e = 0; e < VEC; ++e) a = fmaf(kf[0 + (MM ? 0 : i)].get(e), qv[u][e], a);
#pragma unroll
          for (int x = 1; x < LPRP; x <<= 1) a += __shfl_xor(a, x, 64);
          s[i][u] = valid[i] ? a : -INFINITY;
        }
    }
    // one max decision per head for the UN rows of this lane group
    float muse[G];
    bool up_any = false;
#pragma unroll
    for (int u = 0; u < G; ++u) {
      float mx = s[0][u];
#pragma unroll
      for (int i = 1; i < DEC_UN; ++i) mx = fmaxf(mx, s[i][u]);
      const float m_new = fmaxf(mrun[u], mx);
      const bool up = (m_new - mrun[u]) > DEC_RESCALE_LOG2;   // also true from -inf to a number
      muse[u] = up ? m_new : mrun[u];
      up_any = up_any || up;
    }
    if (__any(up_any)) {
#pragma unroll
      for (int u = 0; u < G; ++u) {
        const float alpha = (muse[u] == mrun[u]) ? 1.f : __builtin_amdgcn_exp2f(mrun[u] - muse[u]);
        lrun[u] *= alpha;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[u][e] *= alpha;
      }
    }
#pragma unroll
    for (int u = 0; u < G; ++u) mrun[u] = muse[u];
#pragma unroll
    for (int i = 0; i < DEC_UN; ++i)
#pragma unroll
      for (int u = 0; u < G; ++u) {
        const float p = valid[i] ? __builtin_amdgcn_exp2f(s[i][u] - muse[u]) : 0.f;
        lrun[u] += p;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[u][e] = fmaf(p, vf[i].get(e), o[u][e]);
      }
  }

  // ---- merge the row slots of the workgroup ----------------------------------------------------
  const int set = wave * KPW + grp;
  if (act) {
#pragma unroll
    for (int u = 0; u < G; ++u) {
      float* dst = sets + (set * G + u) * PW;
#pragma unroll
      for (int e = 0; e < VEC; ++e) dst[off + e] = o[u][e];
      if (sub == 0) {
        dst[D] = mrun[u];
        dst[D + 1] = lrun[u];
      }
    }
  }
  __syncthreads();
  const bool token_wg = !tk.pre && split == n_splits - 1;
  for (int idx = tid; idx < G * PW && !token_wg; idx += DEC_THREADS) {
    const int u = idx / PW, e = idx % PW;
    if (g0 + u >= g) continue;
    float M = -INFINITY;
    for (int s2 = 0; s2 < NSETS; ++s2) M = fmaxf(M, sets[(s2 * G + u) * PW + D]);
    float val;
    if (e == D) {
      val = M;
    } else {
      float acc = 0.f;
      for (int s2 = 0; s2 < NSETS; ++s2) {
        const float ms = sets[(s2 * G + u) * PW + D];
        const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - M);   // empty slots carry nothing
        acc = fmaf(w, sets[(s2 * G + u) * PW + e], acc);     // e == D + 1 merges the sums
      }
      val = acc;
    }
    const int j = m * g + g0 + u;
    part[((int64_t)j * n_splits + split) * PW + e] = val;
  }

  // ---- the new token (last workgroup of the head): its partial for the G heads, and the append ------------------
  if (!token_wg) return;
  __shared__ float ks[D];                              // its key, rotated to position n_keys and rounded as stored
  __shared__ float dots[G][DEC_THREADS / 64];
  if (tid < D) {
    const T* kp = (const T*)tk.k + (int64_t)m * D;
    float ke = Elem<T>::ld(kp + tid);
    if (tab != nullptr) {
      const bool low = tid < D / 2;
      const float kpar = Elem<T>::ld(kp + (low ? tid + D / 2 : tid - D / 2));
      const float2 cs = tab[(int64_t)n_keys * (D / 2) + (low ? tid : tid - D / 2)];
      ke = low ? ke * cs.x - kpar * cs.y : ke * cs.x + kpar * cs.y;
      T rounded;
      Elem<T>::st(&rounded, ke);
      ke = Elem<T>::ld(&rounded);
    }
    ks[tid] = ke;
    if (g0 == 0) {                                     // one launch per step appends
      const int64_t row = ((int64_t)m * cap + n_keys) * D + tid;
      ((T*)tk.K)[row] = kp[tid];
      ((T*)tk.V)[row] = ((const T*)tk.v)[(int64_t)m * D + tid];
      if (tab != nullptr) Elem<T>::st((T*)tk.Kr + row, ke);
      if (tid == 0) {
        tk.P[(int64_t)m * cap + n_keys] = tk.seen;
        if (tk.mark_unscored) tk.S[(int64_t)m * cap + n_keys] = __uint_as_float(0x7fc00000u);   // NaN: ranks last
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < G; ++u) {
    float pr = 0.f;
    if (tid < D) {
      const int j = m * g + min(g0 + u, g - 1);
      const float qe = tab != nullptr ? qs[u * D + tid] : Elem<T>::ld(q + (int64_t)j * D + tid) * c_log2;
      pr = qe * ks[tid];
    }
#pragma unroll
    for (int x = 32; x >= 1; x >>= 1) pr += __shfl_xor(pr, x, 64);
    if (lane == 0) dots[u][wave] = pr;
  }
  __syncthreads();
  for (int idx = tid; idx < G * PW; idx += DEC_THREADS) {
    const int u = idx / PW, e = idx % PW;
    if (g0 + u >= g) continue;
    float val;
    if (e < D) {
      val = Elem<T>::ld((const T*)tk.v + (int64_t)m * D + e);
    } else if (e == D) {
      val = 0.f;
      for (int w2 = 0; w2 < (D + 63) / 64; ++w2) val += dots[u][w2];     // the wavefronts that hold dims, in order
    } else {
      val = 1.f;
    }
    const int j = m * g + g0 + u;
    part[((int64_t)j * n_splits + n_splits - 1) * PW + e] = val;
  }
}

// out[j][:] = sum_s w_s o_s / sum_s w_s l_s with w_s = 2^(m_s - max_s m_s).  One workgroup per head.
// A separate launch on purpose: letting the last workgroup of a head merge behind a device-scope
// fence was measured 3x slower than both kernels together (every workgroup then pays for making its
// partials visible across the eight L2s), while a kernel boundary does that once.
constexpr int DEC_MERGE_THREADS = 1024;
constexpr int DEC_MERGE_PRE = 12;       // vector elements a thread requests before anything else
constexpr int DEC_MERGE_WS = 2048;      // splits whose weights are kept in LDS
template <typename T>
__global__ __launch_bounds__(DEC_MERGE_THREADS) void decode_merge_kernel(const float* __restrict__ part, int n_splits,
                                                                         int d, T* __restrict__ out) {
  // The kernel is a chain of memory latencies, not of bytes (45 KB per head): every load that does not depend on
  // another is requested up front.  Thread (e, r) owns element e of splits r, r + R, ...; the first
  // DEC_MERGE_PRE of them are in flight while the maxima and sums of the splits are reduced.
  __shared__ float red[2 * (DEC_MERGE_THREADS / 64)];
  __shared__ float wsm[DEC_MERGE_WS];
  __shared__ float acc_s[DEC_MERGE_THREADS];
  const int j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pw = d + 2;
  const float* p = part + (int64_t)j * n_splits * pw;
  constexpr int R = DEC_MERGE_THREADS / 128;   // d <= 128
  const int e = tid % 128, r = tid / 128;
  // (addresses are clamped instead of the loads being predicated: a conditional load is a branch, and the wait
  // counters cannot be tracked across it, so every such load would be waited for before the next is issued)
  float pv[DEC_MERGE_PRE];
  const int ec = min(e, d - 1);
#pragma unroll
  for (int i = 0; i < DEC_MERGE_PRE; ++i) pv[i] = p[min(r + i * R, n_splits - 1) * pw + ec];
  // max and sum of split tid in registers; further splits of this thread (more than 1024 splits) are read again
  const float2 ml = *(const float2*)(p + min(tid, n_splits - 1) * pw + d);     // pw and d are even: 8-byte aligned
  const float m0 = tid < n_splits ? ml.x : -INFINITY;
  const float l0 = tid < n_splits ? ml.y : 0.f;
  float mx = m0;
  for (int s = tid + DEC_MERGE_THREADS; s < n_splits; s += DEC_MERGE_THREADS) mx = fmaxf(mx, p[s * pw + d]);
#pragma unroll
  for (int x = 32; x >= 1; x >>= 1) mx = fmaxf(mx, __shfl_xor(mx, x, 64));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  float M = red[0];
#pragma unroll
  for (int i = 1; i < DEC_MERGE_THREADS / 64; ++i) M = fmaxf(M, red[i]);
  // weights w_s = 2^(m_s - M) (a split without keys carries max -inf and weighs 0)
  float ls = 0.f;
  {
    const float w = __builtin_amdgcn_exp2f(m0 - M);
    wsm[tid] = w;
    ls = w * l0;
    for (int s = tid + DEC_MERGE_THREADS; s < n_splits; s += DEC_MERGE_THREADS) {
      const float w2 = __builtin_amdgcn_exp2f(p[s * pw + d] - M);
      if (s < DEC_MERGE_WS) wsm[s] = w2;
      ls = fmaf(w2, p[s * pw + d + 1], ls);
    }
  }
#pragma unroll
  for (int x = 32; x >= 1; x >>= 1) ls += __shfl_xor(ls, x, 64);
  if (lane == 0) red[DEC_MERGE_THREADS / 64 + wave] = ls;
  __syncthreads();                                   // also publishes the weights
  float l = 0.f;
#pragma unroll
  for (int i = 0; i < DEC_MERGE_THREADS / 64; ++i) l += red[DEC_MERGE_THREADS / 64 + i];
  const float inv = 1.f / l;
  float a0 = 0.f;
  if (e < d) {
#pragma unroll
    for (int i = 0; i < DEC_MERGE_PRE; ++i) {
      const int s = r + i * R;
      if (s < n_splits) a0 = fmaf(wsm[s], pv[i], a0);
    }
    for (int s = r + DEC_MERGE_PRE * R; s < n_splits; s += R) {
      const float w = s < DEC_MERGE_WS ? wsm[s] : __builtin_amdgcn_exp2f(p[s * pw + d] - M);
      a0 = fmaf(w, p[s * pw + e], a0);
    }
  }
  acc_s[tid] = a0;
  __syncthreads();
  if (tid < d) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < R; ++i) t += acc_s[tid + i * 128];
    Elem<T>::st(out + (int64_t)j * d + tid, t * inv);
  }
}

// Keys per split.  Tuning::dec_keys (a multiple of 64 in 64 .. 65536) fixes it; otherwise it is chosen per
// launch so that the launch has about 700 workgroups (2.7 per CU), but never under 128 keys, in steps of 64.
// Measured per token, end to end: 8 heads x 16.6K units 24.0 us at 192 keys (25.4 at 256), 32 heads x 8.4K units
// 21.5 us at 384 (22.6 at 256), 8 heads x 6.4K units 14.7 us at 128 (18.6 at 64, 15.6 at 256).
constexpr int DEC_KEYS_MIN = 128;
int decode_keys_per_split(const Dims& D, int n_keys) {
  if (D.tune.dec_keys > 0) return D.tune.dec_keys;
  const int64_t want = ((int64_t)D.h_kv * n_keys + 703) / 704;
  int k = (int)((want + 63) / 64 * 64);
  if (k < DEC_KEYS_MIN) k = DEC_KEYS_MIN;
  if (k > 65536) k = 65536;
  return k;
}

// partials per query head at most: the splits over a full cache at the smallest split size, and the new token's
int decode_max_splits(const Dims& D) {
  const int kmin = D.tune.dec_keys > 0 ? D.tune.dec_keys : DEC_KEYS_MIN;
  return (D.cap + kmin - 1) / kmin + 1;
}

template <typename T, int DD>
static void decode_launch(const Dims& D, const DecodeToken& tk, T* out, float* part, hipStream_t st) {
  const int kpw = decode_keys_per_split(D, tk.n_c);
  const int n_attn = (tk.n_c + tk.pre + kpw - 1) / kpw;   // splits over the units already in the cache (the longest head's)
  const T* Kx = (const T*)(D.rope ? tk.Kr : tk.K);
  const int n_part = n_attn + (tk.pre ? 0 : 1);           // + the workgroup of the new token
  const dim3 grid(n_part, D.h_kv);
  for (int g0 = 0; g0 < D.g; g0 += 4) {
    const int left = D.g - g0;
    if (left >= 3)
      hipLaunchKernelGGL((decode_attn_kernel<T, DD, 4>), grid, dim3(DEC_THREADS), 0, st, Kx, g0, kpw, part, tk);
    else if (left == 2)
      hipLaunchKernelGGL((decode_attn_kernel<T, DD, 2>), grid, dim3(DEC_THREADS), 0, st, Kx, g0, kpw, part, tk);
    else
      hipLaunchKernelGGL((decode_attn_kernel<T, DD, 1>), grid, dim3(DEC_THREADS), 0, st, Kx, g0, kpw, part, tk);
  }
  hipLaunchKernelGGL(decode_merge_kernel<T>, dim3(D.h), dim3(DEC_MERGE_THREADS), 0, st, (const float*)part, n_part, D.d,
                     out);
}

void launch_decode_step(const Dims& D, const void* q, const void* k, const void* v, const CacheBuf& c,
                        const float2* tab, void* out, int n_c, int64_t seen, float scale, float* part, hipStream_t st,
                        bool mark_unscored, const HeadLens* n_c_h, bool pre_appended) {
  DecodeToken tk;
  tk.pre = pre_appended ? 1 : 0;
  tk.q = q; tk.k = k; tk.v = v;
  tk.tab = D.rope ? tab : nullptr;
  tk.K = c.K; tk.V = c.V; tk.Kr = c.Kr; tk.S = c.S; tk.P = c.P;
  tk.g = D.g; tk.cap = D.cap; tk.n_c = n_c; tk.seen = (int)seen; tk.mark_unscored = mark_unscored ? 1 : 0;
  tk.c_log2 = scale * 1.4426950408889634f;
  tk.n_c_h = head_lens_or_common(n_c_h);
#define LOCRET_DEC(DD)                                                                  \
  case DD:                                                                              \
    if (D.bf16) decode_launch<bf16_t, DD>(D, tk, (bf16_t*)out, part, st);               \
    else decode_launch<float, DD>(D, tk, (float*)out, part, st);                        \
    break;
  switch (D.d) {
    LOCRET_DEC(16)
    LOCRET_DEC(32)
    LOCRET_DEC(64)
    LOCRET_DEC(96)
    LOCRET_DEC(128)
  }
#undef LOCRET_DEC
}

}  // namespace locret
