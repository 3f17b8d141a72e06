// Bandwidth-bound cache maintenance kernels for gfx950: rotary table, weight preparation,
// chunk append (Algorithm 1 "Concat") and order-preserving compaction (Algorithm 1 gather).
// Every thread moves 16-byte vectors; a row of d elements is shared by (d/2)/VEC threads, each of
// which owns VEC rotary pairs (i, i + d/2), so the rotated shadow of K is produced from registers.
#include "device_util.h"
#include "kernels.h"

namespace locret {

// ------------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* tab, int cap, int half, int d, double theta) {
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)cap * half) return;
  int pos = (int)(gid / half), i = (int)(gid % half);
  double inv = pow(theta, -2.0 * (double)i / (double)d);
  double a = (double)pos * inv;
  tab[gid] = make_float2((float)cos(a), (float)sin(a));
}

void launch_rope_table(float2* tab, int cap, int d, float theta, hipStream_t st) {
  int64_t n = (int64_t)cap * (d / 2);
  int blocks = (int)((n + 255) / 256);
  hipLaunchKernelGGL(rope_table_kernel, dim3(blocks), dim3(256), 0, st, tab, cap, d / 2, d, (double)theta);
}

// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void prep_w1_kernel(const T* __restrict__ W1, T* __restrict__ W1t, int h, int h_kv, int g, int d,
                               int d_R, int K, int expand) {
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)K * d_R) return;
  int n = (int)(gid % d_R);
  int c = (int)(gid / d_R);
  int hd = h * d;
  float acc;
  if (!expand || c < hd) {
    acc = Elem<T>::ld(W1 + (int64_t)c * d_R + n);
  } else {
    int cc = c - hd;
    int blk = cc / (h_kv * d);          // 0: K block, 1: V block
    int r = cc % (h_kv * d);
    int m = r / d, i = r % d;
    int64_t base = (int64_t)hd * (1 + blk);
    acc = 0.f;
    for (int rep = 0; rep < g; ++rep)
      acc += Elem<T>::ld(W1 + (base + (int64_t)(m * g + rep) * d + i) * d_R + n);
  }
  Elem<T>::st(W1t + (int64_t)n * K + c, acc);
}

template <typename T>
__global__ void prep_w2_kernel(const T* __restrict__ W2, float* __restrict__ W2f, int n) {
  int gid = blockIdx.x * blockDim.x + threadIdx.x;
  if (gid < n) W2f[gid] = Elem<T>::ld(W2 + gid);
}

void launch_prep_weights(const Dims& D, int expand, const void* W1, const void* W2, void* W1t, float* W2f,
                         hipStream_t st) {
  int64_t n1 = (int64_t)D.K * D.d_R;
  int n2 = D.d_R * D.h_kv;
  dim3 b1((unsigned)((n1 + 255) / 256)), b2((unsigned)((n2 + 255) / 256));
  if (D.bf16) {
    hipLaunchKernelGGL(prep_w1_kernel<bf16_t>, b1, dim3(256), 0, st, (const bf16_t*)W1, (bf16_t*)W1t, D.h,
                       D.h_kv, D.g, D.d, D.d_R, D.K, expand);
    hipLaunchKernelGGL(prep_w2_kernel<bf16_t>, b2, dim3(256), 0, st, (const bf16_t*)W2, W2f, n2);
  } else {
    hipLaunchKernelGGL(prep_w1_kernel<float>, b1, dim3(256), 0, st, (const float*)W1, (float*)W1t, D.h,
                       D.h_kv, D.g, D.d, D.d_R, D.K, expand);
    hipLaunchKernelGGL(prep_w2_kernel<float>, b2, dim3(256), 0, st, (const float*)W2, W2f, n2);
  }
}

// ------------------------------------------------------------------------------------------------
// rotate VEC pairs held as (lo, hi) by the table row of `pos`
template <typename T>
__device__ __forceinline__ void rotate_pairs(const Vec16<T>& lo, const Vec16<T>& hi, Vec16<T>& olo, Vec16<T>& ohi,
                                             const float2* __restrict__ tab_row) {
#pragma unroll
  for (int i = 0; i < Vec16<T>::N; ++i) {
    float2 cs = tab_row[i];
    float a = lo.get(i), b = hi.get(i);
    olo.set(i, a * cs.x - b * cs.y);
    ohi.set(i, b * cs.x + a * cs.y);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void append_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                     const T* __restrict__ v, int Tn, int n_c, int seen, int h,
                                                     int h_kv, int d, int cap, T* __restrict__ Kc,
                                                     T* __restrict__ Vc, T* __restrict__ Krc,
                                                     int32_t* __restrict__ Pc, T* __restrict__ qr,
                                                     const float2* __restrict__ tab, int rope, int q_rows,
                                                     float* __restrict__ S_unscored, HeadLens n_c_h) {
  constexpr int VEC = Vec16<T>::N;
  const int half = d / 2;
  const int tpr = half / VEC;
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t row = gid / tpr;
  int part = (int)(gid % tpr);
  const int rows_per_tok = q_rows + 2 * h_kv;   // q_rows = h when queries are rotated here, else 0
  if (row >= (int64_t)Tn * rows_per_tok) return;
  int t = (int)(row / rows_per_tok);
  int r = (int)(row % rows_per_tok);
  int off = part * VEC;
  typedef Vec16<T> V16;
  if (r < q_rows) {
    const T* src = q + ((int64_t)t * h + r) * d;
    V16 lo, hi, olo, ohi;
    lo.raw = *(const decltype(lo.raw)*)(src + off);
    hi.raw = *(const decltype(hi.raw)*)(src + half + off);
    const int n_c_q = head_len(n_c_h, r / (h / h_kv), n_c);   // a query sits behind its own KV head's cache
    rotate_pairs<T>(lo, hi, olo, ohi, tab + (int64_t)(n_c_q + t) * half + off);
    T* dst = qr + ((int64_t)t * h + r) * d;
    *(decltype(lo.raw)*)(dst + off) = olo.raw;
    *(decltype(lo.raw)*)(dst + half + off) = ohi.raw;
    return;
  }
  r -= q_rows;
  const bool is_k = r < h_kv;
  int m = is_k ? r : r - h_kv;
  n_c = head_len(n_c_h, m, n_c);
  const T* src = (is_k ? k : v) + ((int64_t)t * h_kv + m) * d;
  V16 lo, hi;
  lo.raw = *(const decltype(lo.raw)*)(src + off);
  hi.raw = *(const decltype(hi.raw)*)(src + half + off);
  int64_t drow = ((int64_t)m * cap + n_c + t) * d;
  T* dst = (is_k ? Kc : Vc) + drow;
  *(decltype(lo.raw)*)(dst + off) = lo.raw;
  *(decltype(lo.raw)*)(dst + half + off) = hi.raw;
  if (is_k) {
    if (rope) {
      V16 olo, ohi;
      rotate_pairs<T>(lo, hi, olo, ohi, tab + (int64_t)(n_c + t) * half + off);
      *(decltype(lo.raw)*)(Krc + drow + off) = olo.raw;
      *(decltype(lo.raw)*)(Krc + drow + half + off) = ohi.raw;
    }
    if (part == 0) {
      Pc[(int64_t)m * cap + n_c + t] = seen + t;
      if (S_unscored) S_unscored[(int64_t)m * cap + n_c + t] = __uint_as_float(0x7fc00000u);   // NaN: ranks last
    }
  }
}

void launch_append(const Dims& D, const void* q, const void* k, const void* v, int T, int n_c, int64_t seen,
                   const CacheBuf& c, void* qr, const float2* tab, hipStream_t st, bool mark_unscored,
                   const HeadLens* n_c_h) {
  float* Su = mark_unscored ? c.S : nullptr;
  const HeadLens hl = head_lens_or_common(n_c_h);
  const int vec = D.bf16 ? 8 : 4;
  const int tpr = (D.d / 2) / vec;
  const int q_rows = (D.rope && q != nullptr) ? D.h : 0;
  int64_t threads = (int64_t)T * (q_rows + 2 * D.h_kv) * tpr;
  dim3 grid((unsigned)((threads + 255) / 256));
  if (D.bf16)
    launch_kernel(append_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, T, n_c, (int)seen, D.h, D.h_kv, D.d, D.cap, (bf16_t*)c.K, (bf16_t*)c.V,
                       (bf16_t*)c.Kr, c.P, (bf16_t*)qr, tab, D.rope, q_rows, Su, hl);
  else
    launch_kernel(append_kernel<float>, grid, dim3(256), 0, st, (const float*)q, (const float*)k,
                       (const float*)v, T, n_c, (int)seen, D.h, D.h_kv, D.d, D.cap, (float*)c.K, (float*)c.V,
                       (float*)c.Kr, c.P, (float*)qr, tab, D.rope, q_rows, Su, hl);
}

// ------------------------------------------------------------------------------------------------
// Compaction: dst[m][r] = src[m][kept[m][r]].  A thread owns slot r (and VEC rotary pairs of it)
// for ALL KV heads: the rotary table row of slot r is read once and reused for every head, and
// the loads of HB heads are issued together before anything is stored (memory-level parallelism).
// 16-byte loads and stores that bypass the caches' retention: compaction touches every byte once
typedef unsigned int nt_u32x4 __attribute__((ext_vector_type(4)));
template <typename R>
__device__ __forceinline__ R nt_load16(const void* p) {
  static_assert(sizeof(R) == 16, "16-byte lanes");
  nt_u32x4 v = __builtin_nontemporal_load((const nt_u32x4*)p);
  return __builtin_bit_cast(R, v);
}
template <typename R>
__device__ __forceinline__ void nt_store16(void* p, R r) {
  static_assert(sizeof(R) == 16, "16-byte lanes");
  __builtin_nontemporal_store(__builtin_bit_cast(nt_u32x4, r), (nt_u32x4*)p);
}

// RAGGED: head m has keep_h.v[m] rows (head-wise budgets); rows beyond that are neither read nor written.
template <typename T, int HB, bool RAGGED>
__global__ __launch_bounds__(256) void compact_kernel(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                      const float* __restrict__ Ss, const int32_t* __restrict__ Ps,
                                                      T* __restrict__ Kd, T* __restrict__ Vd, T* __restrict__ Krd,
                                                      float* __restrict__ Sd, int32_t* __restrict__ Pd,
                                                      const int32_t* __restrict__ kept, int kept_stride,
                                                      int n_keep, int h_kv, int d, int cap,
                                                      const float2* __restrict__ tab, int rope, int hpb,
                                                      HeadLens keep_h) {
  constexpr int VEC = Vec16<T>::N;
  typedef Vec16<T> V16;
  typedef decltype(V16().raw) raw_t;
  const int half = d / 2;
  const int tpr = half / VEC;
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int r = (int)(gid / tpr);
  const int part = (int)(gid % tpr);
  if (r >= n_keep) return;
  const int off = part * VEC;
  float2 cs[VEC];
  if (rope) {
    const float2* tr = tab + (int64_t)r * half + off;
#pragma unroll
    for (int i = 0; i < VEC; ++i) cs[i] = tr[i];
  }
  const int m_lo = blockIdx.y * hpb, m_hi = min(h_kv, m_lo + hpb);   // this block's KV heads
  for (int m0 = m_lo; m0 < m_hi; m0 += HB) {
    int src[HB];
    V16 klo[HB], khi[HB], vlo[HB], vhi[HB];
#pragma unroll
    for (int u = 0; u < HB; ++u) {
      const int m = min(m0 + u, m_hi - 1);          // spare iterations repeat the last head (stores are skipped)
      if (RAGGED) src[u] = r < keep_h.v[m] ? kept[(int64_t)m * kept_stride + r] : 0;   // row 0: a valid address
      else src[u] = kept[(int64_t)m * kept_stride + r];
    }
#pragma unroll
    for (int u = 0; u < HB; ++u) {
      const int m = min(m0 + u, m_hi - 1);
      const int64_t srow = ((int64_t)m * cap + src[u]) * d;
      klo[u].raw = nt_load16<raw_t>(Ks + srow + off);
      khi[u].raw = nt_load16<raw_t>(Ks + srow + half + off);
      vlo[u].raw = nt_load16<raw_t>(Vs + srow + off);
      vhi[u].raw = nt_load16<raw_t>(Vs + srow + half + off);
    }
#pragma unroll
    for (int u = 0; u < HB; ++u) {
      const int m = m0 + u;
      if (m >= m_hi) break;
      if (RAGGED && r >= keep_h.v[m]) continue;
      const int64_t drow = ((int64_t)m * cap + r) * d;
      nt_store16(Kd + drow + off, klo[u].raw);
      nt_store16(Kd + drow + half + off, khi[u].raw);
      nt_store16(Vd + drow + off, vlo[u].raw);
      nt_store16(Vd + drow + half + off, vhi[u].raw);
      if (rope) {
        V16 olo, ohi;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          float a = klo[u].get(i), b = khi[u].get(i);
          olo.set(i, a * cs[i].x - b * cs[i].y);
          ohi.set(i, b * cs[i].x + a * cs[i].y);
        }
        nt_store16(Krd + drow + off, olo.raw);
        nt_store16(Krd + drow + half + off, ohi.raw);
      }
      if (part == 0) {
        Sd[(int64_t)m * cap + r] = Ss[(int64_t)m * cap + src[u]];
        Pd[(int64_t)m * cap + r] = Ps[(int64_t)m * cap + src[u]];
      }
    }
  }
}

void launch_compact(const Dims& D, const CacheBuf& s, const CacheBuf& t, const int32_t* kept, int kept_stride,
                    int n_keep, const float2* tab, hipStream_t st, const HeadLens* keep_h) {
  const HeadLens hl = head_lens_or_common(keep_h);
  const int vec = D.bf16 ? 8 : 4;
  const int tpr = (D.d / 2) / vec;
  int64_t threads = (int64_t)n_keep * tpr;
  if (threads == 0) return;
  // A thread serves `hpb` KV heads (the rotary-table row is read once for all of them); with many heads
  // and a short cache that leaves too few workgroups, so the heads are then split over blockIdx.y.
  // (config 4, 32 heads x 8192 units: 192 workgroups took 85 us, 768 take 57 us)
  const unsigned gx = (unsigned)((threads + 255) / 256);
  int hpb = D.h_kv;
  while (hpb > 2 && (int64_t)gx * ((D.h_kv + hpb - 1) / hpb) < 768) hpb = (hpb + 1) / 2;
  dim3 grid(gx, (unsigned)((D.h_kv + hpb - 1) / hpb));
  // two heads per batch: enough loads in flight per thread while registers still allow many wavefronts
#define LOCRET_COMPACT(TT, RG)                                                                                   \
  launch_kernel((compact_kernel<TT, 2, RG>), grid, dim3(256), 0, st, (const TT*)s.K, (const TT*)s.V, s.S, s.P, \
                     (TT*)t.K, (TT*)t.V, (TT*)t.Kr, t.S, t.P, kept, kept_stride, n_keep, D.h_kv, D.d, D.cap, tab,   \
                     D.rope, hpb, hl)
  if (D.bf16) { if (hl.ragged) LOCRET_COMPACT(bf16_t, true); else LOCRET_COMPACT(bf16_t, false); }
  else { if (hl.ragged) LOCRET_COMPACT(float, true); else LOCRET_COMPACT(float, false); }
#undef LOCRET_COMPACT
}

}  // namespace locret
