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
// One wavefront per row: lane l owns dims 2l and 2l+1 (one byte of codes); the 16 lanes of a group find its
// minimum and maximum with four butterfly steps.
#include "device_util.h"
#include "kernels.h"

namespace locret {

__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) { return (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16); }

// rotate this lane's two dims of a row held as (x0, x1) per lane, D/2 lanes per row, to position `pos`
template <int D>
__device__ __forceinline__ void rotate_lane_pair(float& x0, float& x1, int lane, const float2* __restrict__ tab, int pos) {
  const int half_lanes = D / 4;                                 // lanes that hold the low half of the row
  const bool low = lane < half_lanes;
  const int partner = low ? lane + half_lanes : lane - half_lanes;
  const float p0 = __shfl(x0, partner & 63, 64), p1 = __shfl(x1, partner & 63, 64);
  if (lane < D / 2) {
    const int i = 2 * (low ? lane : lane - half_lanes);
    const float2 c0 = tab[(int64_t)pos * (D / 2) + i], c1 = tab[(int64_t)pos * (D / 2) + i + 1];
    // low half: a cos - b sin with b the partner; high half: b cos + a sin with a the partner
    x0 = low ? x0 * c0.x - p0 * c0.y : x0 * c0.x + p0 * c0.y;
    x1 = low ? x1 * c1.x - p1 * c1.y : x1 * c1.x + p1 * c1.y;
  }
}

template <int D>
__global__ __launch_bounds__(256) void append_q4_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                        int Tn, int n_c, int seen, int h_kv, int cap,
                                                        uint8_t* __restrict__ Kq, uint8_t* __restrict__ Vq, int qstride,
                                                        bf16_t* __restrict__ Kst, bf16_t* __restrict__ Vst,
                                                        int32_t* __restrict__ P, const float2* __restrict__ tab,
                                                        float* __restrict__ S_unscored) {
  const int lane = threadIdx.x & 63;
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  if (row >= (int64_t)Tn * 2 * h_kv) return;                    // whole wavefronts leave together
  const int t = (int)(row / (2 * h_kv)), r = (int)(row % (2 * h_kv));
  const bool is_k = r < h_kv;
  const int m = is_k ? r : r - h_kv;
  const bool act = lane < D / 2;
  const bf16_t* src = (is_k ? k : v) + ((int64_t)t * h_kv + m) * D;
  const uint32_t two = act ? *(const uint32_t*)(src + 2 * lane) : 0u;
  const float x0 = bf2f((bf16_t)(two & 0xffffu)), x1 = bf2f((bf16_t)(two >> 16));
  float lo = fminf(x0, x1), hi = fmaxf(x0, x1);
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) {
    lo = fminf(lo, __shfl_xor(lo, o, 64));
    hi = fmaxf(hi, __shfl_xor(hi, o, 64));
  }
  float s = bf2f(f2bf(__fdiv_rn(hi - lo, 15.0f)));
  s = s > 0.f ? s : 1.0f;
  const float c0 = fminf(fmaxf(rintf(__fdiv_rn(x0 - lo, s)), 0.f), 15.f);
  const float c1 = fminf(fmaxf(rintf(__fdiv_rn(x1 - lo, s)), 0.f), 15.f);
  uint32_t byte = (uint32_t)c0 | ((uint32_t)c1 << 4);
  // four lanes' bytes into one dword, stored by the first of them
  uint32_t w = byte | (__shfl_down(byte, 1, 64) << 8) | (__shfl_down(byte, 2, 64) << 16) | (__shfl_down(byte, 3, 64) << 24);
  const int64_t slot = (int64_t)m * cap + n_c + t;
  uint8_t* qrow = (is_k ? Kq : Vq) + slot * qstride;
  if (act && (lane & 3) == 0) *(uint32_t*)(qrow + lane) = w;
  if (act && (lane & 15) == 0) *(uint32_t*)(qrow + D / 2 + 4 * (lane >> 4)) = (uint32_t)f2bf(s) | ((uint32_t)f2bf(lo) << 16);
  // staging: the values the row now stands for
  float y0 = fmaf(c0, s, lo), y1 = fmaf(c1, s, lo);
  if (is_k && tab != nullptr) rotate_lane_pair<D>(y0, y1, lane, tab, n_c + t);
  if (act) *(uint32_t*)((is_k ? Kst : Vst) + slot * D + 2 * lane) = pack2_bf16(y0, y1);
  if (is_k && lane == 0) {
    P[slot] = seen + t;
    if (S_unscored) S_unscored[slot] = __uint_as_float(0x7fc00000u);   // NaN: ranks last
  }
}

// dst packed rows r = src packed rows kept[m][r]; staging rows r = their values, K rotated to position r.
template <int D>
__global__ __launch_bounds__(256) void compact_q4_kernel(const uint8_t* __restrict__ Kqs, const uint8_t* __restrict__ Vqs,
                                                         const float* __restrict__ Ss, const int32_t* __restrict__ Ps,
                                                         uint8_t* __restrict__ Kqd, uint8_t* __restrict__ Vqd,
                                                         float* __restrict__ Sd, int32_t* __restrict__ Pd,
                                                         bf16_t* __restrict__ Kst, bf16_t* __restrict__ Vst,
                                                         const int32_t* __restrict__ kept, int kept_stride, int n_keep,
                                                         int h_kv, int cap, int qstride, const float2* __restrict__ tab) {
  const int lane = threadIdx.x & 63;
  const int64_t id = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  if (id >= (int64_t)2 * h_kv * n_keep) return;
  const int r = (int)(id % n_keep);
  const int mk = (int)(id / n_keep);                            // consecutive wavefronts: consecutive slots of one array
  const int m = mk >> 1;
  const bool is_k = (mk & 1) == 0;
  const int src = kept[(int64_t)m * kept_stride + r];
  const int64_t srow = (int64_t)m * cap + src, drow = (int64_t)m * cap + r;
  const int ndw = qstride / 4;
  const uint32_t w = lane < ndw ? *(const uint32_t*)((is_k ? Kqs : Vqs) + srow * qstride + 4 * lane) : 0u;
  if (lane < ndw) *(uint32_t*)((is_k ? Kqd : Vqd) + drow * qstride + 4 * lane) = w;
  const uint32_t byte = (__shfl(w, lane >> 2, 64) >> ((lane & 3) * 8)) & 0xffu;
  const uint32_t par = __shfl(w, (D / 8 + (lane >> 4)) & 63, 64);
  const float s = bf2f((bf16_t)(par & 0xffffu)), lo = bf2f((bf16_t)(par >> 16));
  float y0 = fmaf((float)(byte & 15u), s, lo), y1 = fmaf((float)(byte >> 4), s, lo);
  if (is_k && tab != nullptr) rotate_lane_pair<D>(y0, y1, lane, tab, r);
  if (lane < D / 2) *(uint32_t*)((is_k ? Kst : Vst) + drow * D + 2 * lane) = pack2_bf16(y0, y1);
  if (is_k && lane == 0) {
    Sd[drow] = Ss[srow];
    Pd[drow] = Ps[srow];
  }
}

bool q4_head_dim(int d) { return d == 64 || d == 96 || d == 128; }
int q4_row_bytes(int d) { return d / 2 + 4 * (d / 32); }
int q4_row_stride(int d) { return (q4_row_bytes(d) + 15) / 16 * 16; }

void launch_append_q4(const Dims& D, const void* k, const void* v, int T, int n_c, int64_t seen, const CacheBuf& c,
                      const float2* tab, hipStream_t st, bool mark_unscored) {
  const int64_t rows = (int64_t)T * 2 * D.h_kv;
  const dim3 grid((unsigned)((rows + 3) / 4));
  float* Su = mark_unscored ? c.S : nullptr;
#define LOCRET_Q4A(DD)                                                                                              \
  launch_kernel(append_q4_kernel<DD>, grid, dim3(256), 0, st, (const bf16_t*)k, (const bf16_t*)v, T, n_c,       \
                     (int)seen, D.h_kv, D.cap, (uint8_t*)c.Kq, (uint8_t*)c.Vq, c.qstride, (bf16_t*)c.Kr, (bf16_t*)c.V, \
                     c.P, D.rope ? tab : nullptr, Su)
  if (D.d == 128) LOCRET_Q4A(128); else if (D.d == 96) LOCRET_Q4A(96); else LOCRET_Q4A(64);
#undef LOCRET_Q4A
}

void launch_compact_q4(const Dims& D, const CacheBuf& s, const CacheBuf& t, const int32_t* kept, int kept_stride,
                       int n_keep, const float2* tab, hipStream_t st) {
  const int64_t rows = (int64_t)2 * D.h_kv * n_keep;
  if (rows == 0) return;
  const dim3 grid((unsigned)((rows + 3) / 4));
#define LOCRET_Q4C(DD)                                                                                              \
  launch_kernel(compact_q4_kernel<DD>, grid, dim3(256), 0, st, (const uint8_t*)s.Kq, (const uint8_t*)s.Vq, s.S,  \
                     s.P, (uint8_t*)t.Kq, (uint8_t*)t.Vq, t.S, t.P, (bf16_t*)t.Kr, (bf16_t*)t.V, kept, kept_stride,    \
                     n_keep, D.h_kv, D.cap, s.qstride, D.rope ? tab : nullptr)
  if (D.d == 128) LOCRET_Q4C(128); else if (D.d == 96) LOCRET_Q4C(96); else LOCRET_Q4C(64);
#undef LOCRET_Q4C
}

}  // namespace locret
