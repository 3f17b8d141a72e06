// Plain-VALU float kernels for the chunk attention (Eq. 1) and the retaining head (Section 3.3).
// They serve the float32 configuration (where bf16 matrix cores would break the 1e-5 bar) and any
// head_dim the MFMA kernels do not cover.  All arithmetic is float32 with float32 accumulation;
// storage may be float or bf16.
#include "device_util.h"
#include "kernels.h"

namespace locret {

// ------------------------------------------------------------------------------------------------
// Attention.  Workgroup = 256 threads = 32 query rows x 8 column threads, one query head.
// Key tiles of 64 slots are staged in LDS; thread (r, c) computes the logits of keys c, c+8, ...
// with the whole query row in registers, then owns output dims [c*D/8, (c+1)*D/8).
// ------------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_simple_kernel(const T* __restrict__ q, const T* __restrict__ Kx,
                                                          const T* __restrict__ V, T* __restrict__ out, int Tn,
                                                          int h, int g, int cap, int n_c_common, float scale,
                                                          HeadLens n_c_h) {
  constexpr int KT = (D > 64) ? 32 : 64;   // keeps K, V, P tiles under 64 KB of LDS
  constexpr int NI = KT / 8;               // keys per thread per tile
  constexpr int DP = D + 4;           // padded row (floats)
  constexpr int DC = D / 8;           // output dims per thread
  __shared__ float Ks[KT * DP];
  __shared__ float Vs[KT * DP];
  __shared__ float Ps[32 * (KT + 1)];

  const int tid = threadIdx.x;
  const int r = tid >> 3, c = tid & 7;
  const int j = blockIdx.y;
  const int m = j / g;
  const int n_c = head_len(n_c_h, m, n_c_common);
  const int t0 = blockIdx.x * 32;
  const int t = t0 + r;
  const bool row_ok = t < Tn;
  const int t_last = min(Tn - 1, t0 + 31);
  const int n_keys = n_c + t_last + 1;          // slots any row of this tile may see
  const int my_last = n_c + t;                  // last visible slot of this row

  float qreg[D];
  {
    const T* qp = q + ((int64_t)(row_ok ? t : t_last) * h + j) * D;
#pragma unroll
    for (int e = 0; e < D; ++e) qreg[e] = Elem<T>::ld(qp + e) * scale;
  }
  float acc[DC];
#pragma unroll
  for (int e = 0; e < DC; ++e) acc[e] = 0.f;
  float mrun = -INFINITY, lrun = 0.f;

  const T* Kb = Kx + (int64_t)m * cap * D;
  const T* Vb = V + (int64_t)m * cap * D;

  for (int k0 = 0; k0 < n_keys; k0 += KT) {
    __syncthreads();
    for (int idx = tid; idx < KT * D; idx += 256) {
      int kk = idx / D, e = idx % D;
      int slot = k0 + kk;
      float kv = 0.f, vv = 0.f;
      if (slot < n_keys) {
        kv = Elem<T>::ld(Kb + (int64_t)slot * D + e);
        vv = Elem<T>::ld(Vb + (int64_t)slot * D + e);
      }
      Ks[kk * DP + e] = kv;
      Vs[kk * DP + e] = vv;
    }
    __syncthreads();
    float sv[NI];
    float tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int kk = c + 8 * i;
      const float* kp = Ks + kk * DP;
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < D; e += 4) {
        float4 k4 = *(const float4*)(kp + e);
        dot = fmaf(qreg[e], k4.x, dot);
        dot = fmaf(qreg[e + 1], k4.y, dot);
        dot = fmaf(qreg[e + 2], k4.z, dot);
        dot = fmaf(qreg[e + 3], k4.w, dot);
      }
      bool vis = (k0 + kk) <= my_last;
      sv[i] = vis ? dot : -INFINITY;
      tmax = fmaxf(tmax, sv[i]);
    }
    // row max across the 8 column threads (consecutive lanes)
    tmax = fmaxf(tmax, __shfl_xor(tmax, 1, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 2, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 4, 64));
    float mnew = fmaxf(mrun, tmax);      // finite: slot k0 <= n_c <= my_last is always visible in tile 0
    float alpha = expf(mrun - mnew);     // exp(-inf) = 0 on the first tile
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float p = expf(sv[i] - mnew);
      psum += p;
      Ps[r * (KT + 1) + c + 8 * i] = p;
    }
    psum += __shfl_xor(psum, 1, 64);
    psum += __shfl_xor(psum, 2, 64);
    psum += __shfl_xor(psum, 4, 64);
    lrun = lrun * alpha + psum;
    mrun = mnew;
#pragma unroll
    for (int e = 0; e < DC; ++e) acc[e] *= alpha;
    __syncthreads();
    const float* pp = Ps + r * (KT + 1);
    for (int kk = 0; kk < KT; ++kk) {
      float p = pp[kk];
      const float* vp = Vs + kk * DP + c * DC;
#pragma unroll
      for (int e = 0; e < DC; ++e) acc[e] = fmaf(p, vp[e], acc[e]);
    }
  }
  if (row_ok) {
    T* op = out + ((int64_t)t * h + j) * D + c * DC;
    float inv = 1.f / lrun;
#pragma unroll
    for (int e = 0; e < DC; ++e) Elem<T>::st(op + e, acc[e] * inv);
  }
}

template <typename T>
static void attn_simple_dispatch(const Dims& D, const void* q, const void* Kx, const void* V, void* out, int Tn,
                                 int n_c, float scale, hipStream_t st, const HeadLens& hl) {
  dim3 grid((Tn + 31) / 32, D.h);
#define LOCRET_ATTN_CASE(DD)                                                                                    \
  case DD:                                                                                                      \
    hipLaunchKernelGGL((attn_simple_kernel<T, DD>), grid, dim3(256), 0, st, (const T*)q, (const T*)Kx,          \
                       (const T*)V, (T*)out, Tn, D.h, D.g, D.cap, n_c, scale, hl);                              \
    break;
  switch (D.d) {
    LOCRET_ATTN_CASE(16)
    LOCRET_ATTN_CASE(32)
    LOCRET_ATTN_CASE(64)
    LOCRET_ATTN_CASE(96)
    LOCRET_ATTN_CASE(128)
    default: break;
  }
#undef LOCRET_ATTN_CASE
}

void launch_attention_simple(const Dims& D, const void* q, const void* Kx, const void* V, void* out, int T,
                             int n_c, float scale, hipStream_t st, const HeadLens* n_c_h) {
  const HeadLens hl = head_lens_or_common(n_c_h);
  if (D.bf16) attn_simple_dispatch<bf16_t>(D, q, Kx, V, out, T, n_c, scale, st, hl);
  else attn_simple_dispatch<float>(D, q, Kx, V, out, T, n_c, scale, st, hl);
}

// ------------------------------------------------------------------------------------------------
// Retaining head.  Tile = 64 tokens x 64 hidden units per 256-thread workgroup, k-step 16;
// thread (ty, tx) accumulates a 4x4 block.  The [q;k;v] input row is read in place from the three
// tensors.  SiLU and the product with W2 happen in the epilogue; each workgroup writes its
// hidden-block partial  part[nb][m][t]  (summed later in a fixed order).
// ------------------------------------------------------------------------------------------------
constexpr int SC_TM = 64, SC_TN = 64, SC_TK = 16;

template <typename T>
__global__ __launch_bounds__(256) void score_simple_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                           const T* __restrict__ v, int Tn, int hd, int kvd,
                                                           const T* __restrict__ W1t, const float* __restrict__ W2f,
                                                           int K, int d_R, int h_kv, float* __restrict__ part,
                                                           int part_T) {
  __shared__ float As[SC_TK][SC_TM + 4];
  __shared__ float Bs[SC_TK][SC_TN + 4];
  __shared__ float Hs[SC_TM][SC_TN + 1];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int t0 = blockIdx.x * SC_TM;
  const int nb = blockIdx.y;
  const int n0 = nb * SC_TN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += SC_TK) {
    // the 16 input columns of this step lie in one of q, k, v (hd and kvd are multiples of 16)
    const T* src; int cw, c0;
    if (k0 < hd) { src = q; cw = hd; c0 = k0; }
    else if (k0 < hd + kvd) { src = k; cw = kvd; c0 = k0 - hd; }
    else { src = v; cw = kvd; c0 = k0 - hd - kvd; }
    __syncthreads();
    for (int idx = tid; idx < SC_TM * SC_TK; idx += 256) {
      int row = idx / SC_TK, kk = idx % SC_TK;
      int t = t0 + row;
      As[kk][row] = (t < Tn) ? Elem<T>::ld(src + (int64_t)t * cw + c0 + kk) : 0.f;
      int n = n0 + row;
      Bs[kk][row] = (n < d_R) ? Elem<T>::ld(W1t + (int64_t)n * K + k0 + kk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < SC_TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) acc[i][jn] = fmaf(a[i], b[jn], acc[i][jn]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) {
      float z = acc[i][jn];
      Hs[ty * 4 + i][tx * 4 + jn] = z / (1.f + expf(-z));
    }
  __syncthreads();
  for (int idx = tid; idx < SC_TM * h_kv; idx += 256) {
    int row = idx % SC_TM, m = idx / SC_TM;
    float sum = 0.f;
    const int hh_end = min(SC_TN, d_R - n0);
    for (int hh = 0; hh < hh_end; ++hh) sum = fmaf(Hs[row][hh], W2f[(int64_t)(n0 + hh) * h_kv + m], sum);
    int t = t0 + row;
    if (t < Tn) part[((int64_t)nb * h_kv + m) * part_T + t] = sum;
  }
}

int score_parts_simple(const Dims& D) { return (D.d_R + SC_TN - 1) / SC_TN; }

void launch_score_simple(const Dims& D, const void* q, const void* k, const void* v, int T, const void* W1t,
                         const float* W2f, float* part, hipStream_t st) {
  dim3 grid((T + SC_TM - 1) / SC_TM, (D.d_R + SC_TN - 1) / SC_TN);
  const int hd = D.h * D.d, kvd = D.h_kv * D.d;
  if (D.bf16)
    launch_kernel(score_simple_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, T, hd, kvd, (const bf16_t*)W1t, W2f, D.K, D.d_R, D.h_kv, part, T);
  else
    launch_kernel(score_simple_kernel<float>, grid, dim3(256), 0, st, (const float*)q, (const float*)k,
                       (const float*)v, T, hd, kvd, (const float*)W1t, W2f, D.K, D.d_R, D.h_kv, part, T);
}

// ------------------------------------------------------------------------------------------------
__global__ void score_reduce_kernel(const float* __restrict__ part, int n_parts, int part_T, int h_kv, int Tn,
                                    float* __restrict__ S, int cap, int n_c, float* __restrict__ out,
                                    HeadLens n_c_h) {
  int gid = blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= h_kv * Tn) return;
  int m = gid / Tn, t = gid % Tn;
  float sum = part[(int64_t)m * part_T + t];   // a single part is copied bit for bit (-0 stays -0)
  for (int p = 1; p < n_parts; ++p) sum += part[((int64_t)p * h_kv + m) * part_T + t];
  if (S) S[(int64_t)m * cap + head_len(n_c_h, m, n_c) + t] = sum;
  if (out) out[(int64_t)m * Tn + t] = sum;
}

void launch_score_reduce(const float* part, int n_parts, int part_T, int h_kv, int T, float* S, int cap, int n_c,
                         float* out, hipStream_t st, const HeadLens* n_c_h) {
  int n = h_kv * T;
  launch_kernel(score_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, st, part, n_parts, part_T, h_kv, T,
                     S, cap, n_c, out, head_lens_or_common(n_c_h));
}

}  // namespace locret
