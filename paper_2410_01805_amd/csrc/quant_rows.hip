// 4-bit cache rows (appendix "Orthogonality to Other Methods": Locret combined with 4-bit KV-cache quantization).
//
// Row format (this build's reading; the paper names a third-party quantizer and gives no format): a unit's K or V
// row of d bf16 values is cut into groups of 32 consecutive dims; a group stores asymmetric 4-bit codes
//   code = clamp(round_half_even((x - lo) / s), 0, 15),  lo = min of the group,  s = bf16((max - min) / 15), s = 1 if 0,
// decided in float32, and the row is d/2 code bytes (dim 2i in the low nibble, 2i+1 in the high one) followed by
// (s, lo) as two little-endian bf16 per group; rows are padded to a multiple of 16 bytes in the cache.  A unit is
// self-contained, so eviction moves packed rows unchanged.  K is quantized un-rotated.
//
// The persistent cache (both copies) holds packed rows only.  What attention reads is a single bf16 staging
// array per operand: the dequantized value lo + code * s of every row, K rotated to its slot's position.  It is a
// pure function of the live packed copy: append and compaction write both, so a step still touches each row once.
//
// Both kernels move 16 bytes per lane: a row is shared by head_dim/16 lanes, each owning two pieces of 8 dims that
// are rotary partners, and a thread serves several KV heads so that the rotary-table entries of a position are
// read once.
#include "device_util.h"
#include "kernels.h"

namespace locret {


__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) { return (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16); }

typedef unsigned int q4_u32x4 __attribute__((ext_vector_type(4)));

// A row of D bf16 values is shared by NP = D/16 lanes (a power-of-two block of NPP lanes is reserved for it); lane p
// owns two pieces of 8 dims, [8p, 8p+8) and [D/2 + 8p, D/2 + 8p + 8): eight rotary pairs (i, i + D/2).  Piece ids
// run 0 .. 2 NP - 1 in dim order (piece q = dims [8q, 8q+8)); a quantization group is four consecutive pieces.
template <int D>
struct Q4Lanes {
  static constexpr int NP = D / 16;
  static constexpr int NPP = NP <= 4 ? 4 : 8;
};

// min and max of the group that piece `piece` belongs to, gathered from the lanes of the row (lane block starts at
// lane `base`): every lane offers the (min, max) of its two pieces.
template <int D>
__device__ __forceinline__ void group_min_max(int piece, int base, float mn0, float mx0, float mn1, float mx1, float& lo, float& hi) {
  constexpr int NP = Q4Lanes<D>::NP;
  const int g = piece >> 2;
  lo = INFINITY;
  hi = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int q = 4 * g + j;                      // a member piece: slot q / NP of lane q % NP
    const int src = base + q % NP;
    const float a0 = __shfl(mn0, src, 64), a1 = __shfl(mn1, src, 64);
    const float b0 = __shfl(mx0, src, 64), b1 = __shfl(mx1, src, 64);
    lo = fminf(lo, q / NP ? a1 : a0);
    hi = fmaxf(hi, q / NP ? b1 : b0);
  }
}

// codes of 8 values against (lo, s); returns the packed dword (dim e in nibble e) and leaves the dequantized values
__device__ __forceinline__ uint32_t quant8(float (&x)[8], float lo, float s) {
  uint32_t w = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float c = fminf(fmaxf(rintf(__fdiv_rn(x[e] - lo, s)), 0.f), 15.f);
    w |= (uint32_t)c << (4 * e);
    x[e] = fmaf(c, s, lo);
  }
  return w;
}

__device__ __forceinline__ void unpack8_bf16(q4_u32x4 v, float (&x)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = bf2f((bf16_t)(v[i] & 0xffffu));
    x[2 * i + 1] = bf2f((bf16_t)(v[i] >> 16));
  }
}
__device__ __forceinline__ q4_u32x4 pack8_bf16(const float (&x)[8]) {
  q4_u32x4 r = {pack2_bf16(x[0], x[1]), pack2_bf16(x[2], x[3]), pack2_bf16(x[4], x[5]), pack2_bf16(x[6], x[7])};
  return r;
}

// Append: thread (t, p) quantizes its two pieces of the K row and of the V row of token t for the KV heads of its
// block, writes the code dwords and (first lane of every group) the group's (scale, minimum), and the staging
// values: what the row now stands for, K rotated to position n_c + t.
template <int D>
__global__ __launch_bounds__(256) void append_q4_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                        int Tn, int n_c, int seen, int h_kv, int cap,
                                                        uint8_t* __restrict__ Kq, uint8_t* __restrict__ Vq, int qstride,
                                                        bf16_t* __restrict__ Kst, bf16_t* __restrict__ Vst,
                                                        int32_t* __restrict__ P, const float2* __restrict__ tab,
                                                        float* __restrict__ S_unscored, int hpb) {
  constexpr int NP = Q4Lanes<D>::NP, NPP = Q4Lanes<D>::NPP;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int t_raw = (int)(gid / NPP), p_raw = (int)(gid % NPP);
  // threads past the chunk and the spare lanes of a block stay in the shuffles (on clamped indices), write nothing
  const bool act = t_raw < Tn && p_raw < NP;
  const int t = min(t_raw, Tn - 1), p = min(p_raw, NP - 1);
  const int base = (threadIdx.x & 63) - p_raw;                  // first lane of the row's block
  float2 cs[8];
  if (tab != nullptr) {
    const float2* tr = tab + (int64_t)(n_c + t) * (D / 2) + 8 * p;
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = tr[e];
  }
  const int m_lo = blockIdx.y * hpb, m_hi = min(h_kv, m_lo + hpb);
  for (int m = m_lo; m < m_hi; ++m) {
    const int64_t slot = (int64_t)m * cap + n_c + t;
#pragma unroll
    for (int kv = 0; kv < 2; ++kv) {
      const bf16_t* src = (kv == 0 ? k : v) + ((int64_t)t * h_kv + m) * D;
      float a[8], b[8];
      unpack8_bf16(*(const q4_u32x4*)(src + 8 * p), a);
      unpack8_bf16(*(const q4_u32x4*)(src + D / 2 + 8 * p), b);
      float mn0 = a[0], mx0 = a[0], mn1 = b[0], mx1 = b[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) {
        mn0 = fminf(mn0, a[e]); mx0 = fmaxf(mx0, a[e]);
        mn1 = fminf(mn1, b[e]); mx1 = fmaxf(mx1, b[e]);
      }
      float lo0, hi0, lo1, hi1;
      group_min_max<D>(p, base, mn0, mx0, mn1, mx1, lo0, hi0);
      group_min_max<D>(NP + p, base, mn0, mx0, mn1, mx1, lo1, hi1);
      float s0 = bf2f(f2bf(__fdiv_rn(hi0 - lo0, 15.0f))), s1 = bf2f(f2bf(__fdiv_rn(hi1 - lo1, 15.0f)));
      s0 = s0 > 0.f ? s0 : 1.0f;
      s1 = s1 > 0.f ? s1 : 1.0f;
      const uint32_t w0 = quant8(a, lo0, s0), w1 = quant8(b, lo1, s1);     // a, b now hold the dequantized values
      if (kv == 0 && tab != nullptr) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float lo = a[e] * cs[e].x - b[e] * cs[e].y, hi = b[e] * cs[e].x + a[e] * cs[e].y;
          a[e] = lo;
          b[e] = hi;
        }
      }
      if (act) {
        uint8_t* qrow = (kv == 0 ? Kq : Vq) + slot * qstride;
        *(uint32_t*)(qrow + 4 * p) = w0;
        *(uint32_t*)(qrow + D / 4 + 4 * p) = w1;
        if ((p & 3) == 0) *(uint32_t*)(qrow + D / 2 + 4 * (p >> 2)) = (uint32_t)f2bf(s0) | ((uint32_t)f2bf(lo0) << 16);
        if (((NP + p) & 3) == 0) *(uint32_t*)(qrow + D / 2 + 4 * ((NP + p) >> 2)) = (uint32_t)f2bf(s1) | ((uint32_t)f2bf(lo1) << 16);
        bf16_t* st = (kv == 0 ? Kst : Vst) + slot * D;
        *(q4_u32x4*)(st + 8 * p) = pack8_bf16(a);
        *(q4_u32x4*)(st + D / 2 + 8 * p) = pack8_bf16(b);
      }
    }
    if (act && p == 0) {
      P[slot] = seen + t;
      if (S_unscored) S_unscored[slot] = __uint_as_float(0x7fc00000u);   // NaN: ranks last
    }
  }
}

// Compaction of packed rows: dst packed rows r = src packed rows kept[m][r]; staging rows r = their values, K rotated
// to position r.  A thread owns slot r and the dims [8p, 8p+8) and [D/2 + 8p, D/2 + 8p + 8) of it, i.e. eight rotary
// pairs, for ALL KV heads of its block (HB heads per batch of loads): the rotary-table entries of slot r are read
// once, the staging stores are 16 bytes per lane, and the first row_stride/16 lanes of a row also move the packed
// row itself, 16 bytes each.
__device__ __forceinline__ void dequant8(uint32_t codes, uint32_t par, float (&x)[8]) {
  const float s = bf2f((bf16_t)(par & 0xffffu)), lo = bf2f((bf16_t)(par >> 16));
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = fmaf((float)((codes >> (4 * e)) & 15u), s, lo);
}

template <int D, int HB>
__global__ __launch_bounds__(256) void compact_q4_kernel(const uint8_t* __restrict__ Kqs, const uint8_t* __restrict__ Vqs,
                                                         const float* __restrict__ Ss, const int32_t* __restrict__ Ps,
                                                         uint8_t* __restrict__ Kqd, uint8_t* __restrict__ Vqd,
                                                         float* __restrict__ Sd, int32_t* __restrict__ Pd,
                                                         bf16_t* __restrict__ Kst, bf16_t* __restrict__ Vst,
                                                         const int32_t* __restrict__ kept, int kept_stride, int n_keep,
                                                         int h_kv, int cap, int qstride, const float2* __restrict__ tab,
                                                         int hpb) {
  constexpr int NP = D / 16;                                    // lanes per row
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int r = (int)(gid / NP), p = (int)(gid % NP);
  if (r >= n_keep) return;
  const int g0 = (8 * p) / 32, g1 = (D / 2 + 8 * p) / 32;       // quantization groups of the lane's two pieces
  const bool mover = p < qstride / 16;                          // also moves 16 bytes of every packed row
  float2 cs[8];
  if (tab != nullptr) {
    const float2* tr = tab + (int64_t)r * (D / 2) + 8 * p;
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = tr[e];
  }
  const int m_lo = blockIdx.y * hpb, m_hi = min(h_kv, m_lo + hpb);
  for (int m0 = m_lo; m0 < m_hi; m0 += HB) {
    int src[HB];
    uint32_t kc0[HB], kc1[HB], kp0[HB], kp1[HB], vc0[HB], vc1[HB], vp0[HB], vp1[HB];
    q4_u32x4 kmv[HB], vmv[HB];
#pragma unroll
    for (int u = 0; u < HB; ++u) src[u] = kept[(int64_t)min(m0 + u, m_hi - 1) * kept_stride + r];   // spare iterations repeat the last head
#pragma unroll
    for (int u = 0; u < HB; ++u) {
      const int m = min(m0 + u, m_hi - 1);
      const uint8_t* kr = Kqs + ((int64_t)m * cap + src[u]) * qstride;
      const uint8_t* vr = Vqs + ((int64_t)m * cap + src[u]) * qstride;
      kc0[u] = *(const uint32_t*)(kr + 4 * p);
      kc1[u] = *(const uint32_t*)(kr + D / 4 + 4 * p);
      kp0[u] = *(const uint32_t*)(kr + D / 2 + 4 * g0);
      kp1[u] = *(const uint32_t*)(kr + D / 2 + 4 * g1);
      vc0[u] = *(const uint32_t*)(vr + 4 * p);
      vc1[u] = *(const uint32_t*)(vr + D / 4 + 4 * p);
      vp0[u] = *(const uint32_t*)(vr + D / 2 + 4 * g0);
      vp1[u] = *(const uint32_t*)(vr + D / 2 + 4 * g1);
      if (mover) {
        kmv[u] = *(const q4_u32x4*)(kr + 16 * p);
        vmv[u] = *(const q4_u32x4*)(vr + 16 * p);
      }
    }
#pragma unroll
    for (int u = 0; u < HB; ++u) {
      const int m = m0 + u;
      if (m >= m_hi) break;
      const int64_t drow = (int64_t)m * cap + r;
      if (mover) {
        __builtin_nontemporal_store(kmv[u], (q4_u32x4*)(Kqd + drow * qstride + 16 * p));
        __builtin_nontemporal_store(vmv[u], (q4_u32x4*)(Vqd + drow * qstride + 16 * p));
      }
      float a[8], bq[8];
      dequant8(kc0[u], kp0[u], a);
      dequant8(kc1[u], kp1[u], bq);
      if (tab != nullptr) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float lo = a[e] * cs[e].x - bq[e] * cs[e].y, hi = bq[e] * cs[e].x + a[e] * cs[e].y;
          a[e] = lo;
          bq[e] = hi;
        }
      }
      __builtin_nontemporal_store(pack8_bf16(a), (q4_u32x4*)(Kst + drow * D + 8 * p));
      __builtin_nontemporal_store(pack8_bf16(bq), (q4_u32x4*)(Kst + drow * D + D / 2 + 8 * p));
      dequant8(vc0[u], vp0[u], a);
      dequant8(vc1[u], vp1[u], bq);
      __builtin_nontemporal_store(pack8_bf16(a), (q4_u32x4*)(Vst + drow * D + 8 * p));
      __builtin_nontemporal_store(pack8_bf16(bq), (q4_u32x4*)(Vst + drow * D + D / 2 + 8 * p));
      if (p == 0) {
        Sd[drow] = Ss[(int64_t)m * cap + src[u]];
        Pd[drow] = Ps[(int64_t)m * cap + src[u]];
      }
    }
  }
}

bool q4_head_dim(int d) { return d == 64 || d == 96 || d == 128; }
int q4_row_bytes(int d) { return d / 2 + 4 * (d / 32); }
int q4_row_stride(int d) { return (q4_row_bytes(d) + 15) / 16 * 16; }

void launch_append_q4(const Dims& D, const void* k, const void* v, int T, int n_c, int64_t seen, const CacheBuf& c,
                      const float2* tab, hipStream_t st, bool mark_unscored) {
  const int npp = D.d / 16 <= 4 ? 4 : 8;
  const int64_t threads = (int64_t)T * npp;
  const unsigned gx = (unsigned)((threads + 255) / 256);
  int hpb = D.h_kv;
  while (hpb > 1 && (int64_t)gx * ((D.h_kv + hpb - 1) / hpb) < 768) hpb = (hpb + 1) / 2;
  const dim3 grid(gx, (unsigned)((D.h_kv + hpb - 1) / hpb));
  float* Su = mark_unscored ? c.S : nullptr;
#define LOCRET_Q4A(DD)                                                                                              \
  launch_kernel(append_q4_kernel<DD>, grid, dim3(256), 0, st, (const bf16_t*)k, (const bf16_t*)v, T, n_c,            \
                (int)seen, D.h_kv, D.cap, (uint8_t*)c.Kq, (uint8_t*)c.Vq, c.qstride, (bf16_t*)c.Kr, (bf16_t*)c.V,    \
                c.P, D.rope ? tab : nullptr, Su, hpb)
  if (D.d == 128) LOCRET_Q4A(128); else if (D.d == 96) LOCRET_Q4A(96); else LOCRET_Q4A(64);
#undef LOCRET_Q4A
}

void launch_compact_q4(const Dims& D, const CacheBuf& s, const CacheBuf& t, const int32_t* kept, int kept_stride,
                       int n_keep, const float2* tab, hipStream_t st) {
  const int64_t threads = (int64_t)n_keep * (D.d / 16);
  if (threads == 0) return;
  // as in the bf16 compaction: a thread serves `hpb` KV heads, fewer when that leaves too few workgroups
  const unsigned gx = (unsigned)((threads + 255) / 256);
  int hpb = D.h_kv;
  while (hpb > 2 && (int64_t)gx * ((D.h_kv + hpb - 1) / hpb) < 768) hpb = (hpb + 1) / 2;
  const dim3 grid(gx, (unsigned)((D.h_kv + hpb - 1) / hpb));
#define LOCRET_Q4C(DD)                                                                                              \
  launch_kernel((compact_q4_kernel<DD, 2>), grid, dim3(256), 0, st, (const uint8_t*)s.Kq, (const uint8_t*)s.Vq, s.S,  \
                s.P, (uint8_t*)t.Kq, (uint8_t*)t.Vq, t.S, t.P, (bf16_t*)t.Kr, (bf16_t*)t.V, kept, kept_stride,       \
                n_keep, D.h_kv, D.cap, s.qstride, D.rope ? tab : nullptr, hpb)
  if (D.d == 128) LOCRET_Q4C(128); else if (D.d == 96) LOCRET_Q4C(96); else LOCRET_Q4C(64);
#undef LOCRET_Q4C
}

}  // namespace locret
