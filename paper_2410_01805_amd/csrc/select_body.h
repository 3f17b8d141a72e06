// Exact top-k selection over the retaining-head scores of one KV head with the keys held in registers
// (the body of select_reg_kernel, also run by workgroups of the head_dim-128 attention launch): see
// select.hip for the method.  NT threads (512 or 1024), MAXR keys per thread, MAXR * 64 * (NT / 64) >= the
// number of candidates.  smem: 256 * SEL_REP + 256 + 2 * (NT / 64) + 2 words.
#pragma once
#include "device_util.h"
#include "kernels.h"

namespace locret {

__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN: below every number
  if (u == 0x80000000u) u = 0u;                     // -0 ties with +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// The selection's sizes for KV head m: the common ones, or with head-wise budgets the head's own
// (the stabilizers and the pinned prefix clamped to what this head holds).
struct HeadSel { int L, n_keep, n_stab, n_pin; };
__device__ __forceinline__ HeadSel head_sel(const SelectArgs& a, int m) {
  HeadSel r;
  r.L = head_len(a.L_h, m, a.L);
  r.n_keep = head_len(a.keep_h, m, a.n_keep);
  r.n_stab = min(a.n_stab, r.L);
  r.n_pin = min(a.n_pin, r.L - r.n_stab);
  return r;
}

constexpr int SEL_REP = 32;    // counter replicas per bin (= LDS banks)

template <int MAXR, int NT>
__device__ __forceinline__ void select_reg_body(const SelectArgs& a, int m, uint32_t* smem) {
  static_assert(NT == 512 || NT == 1024, "threads per bin in the replica sum");
  constexpr int NWAVES = NT / 64;
  uint32_t* hist = smem;                       // [256][SEL_REP]
  uint32_t* tot = hist + 256 * SEL_REP;        // [256]
  uint32_t* wsum = tot + 256;                  // [2][NWAVES]
  uint32_t* bc = wsum + 2 * NWAVES;            // [2]
  const int tid = threadIdx.x;
  const HeadSel hs = head_sel(a, m);
  const float* s = a.S + (int64_t)m * a.cap + hs.n_pin;   // candidate c is unit n_pin + c
  if (a.part != nullptr) {
    const int red_n_c = hs.L - a.red_T;
    // the chunk's scores first: the same sum, in the same order, as score_reduce_kernel
    for (int t = tid; t < a.red_T; t += NT) {
      float sum = a.part[(int64_t)m * a.part_T + t];   // a single part is copied bit for bit (-0 stays -0)
      for (int p = 1; p < a.n_parts; ++p) sum += a.part[((int64_t)p * a.h_kv + m) * a.part_T + t];
      a.S_w[(int64_t)m * a.cap + red_n_c + t] = sum;
      if (a.red_out) a.red_out[(int64_t)m * a.red_T + t] = sum;
    }
    __syncthreads();   // workgroup-scope release/acquire: the keys below are read back from S by other threads
  }
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int L = hs.L, n_pin = hs.n_pin;
  const int n_cand = L - hs.n_stab - n_pin;
  const int kk = hs.n_keep - hs.n_stab - n_pin;
  const int wseg = ((n_cand + NWAVES - 1) / NWAVES + 63) & ~63;     // <= MAXR * 64 (checked by the host)
  const int w_lo = wave * wseg;
  const int w_hi = min(n_cand, w_lo + wseg);
  const int first = w_lo + lane;
  const int nvalid = first < w_hi ? (w_hi - first + 63) >> 6 : 0;        // this thread's keys: rounds 0 .. nvalid-1

  uint32_t k[MAXR];
  {
    float f[MAXR];
#pragma unroll
    for (int j = 0; j < MAXR; ++j) f[j] = (j < nvalid) ? s[first + j * 64] : 0.f;
#pragma unroll
    for (int j = 0; j < MAXR; ++j) k[j] = score_key(f[j]);
  }

  uint32_t tau, need_eq;
  if (kk >= n_cand) {
    tau = 0u; need_eq = 0xffffffffu;
  } else if (kk == 0) {
    tau = 0xffffffffu; need_eq = 0u;
  } else {
    uint32_t prefix = 0u, mask = 0u, remaining = (uint32_t)kk;
    const int rep = lane & (SEL_REP - 1);
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      for (int i = tid; i < 256 * SEL_REP; i += NT) hist[i] = 0u;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < MAXR; ++j)
        if (j < nvalid && (k[j] & mask) == prefix) atomicAdd(&hist[((k[j] >> shift) & 255u) * SEL_REP + rep], 1u);
      __syncthreads();
      {
        constexpr int TPB = NT / 256;            // threads per bin: 4 or 2
        const int bin = tid / TPB, part = tid % TPB;
        uint32_t sum = 0;
#pragma unroll
        for (int r = 0; r < SEL_REP / TPB; ++r) sum += hist[bin * SEL_REP + part * (SEL_REP / TPB) + r];
        sum += __shfl_xor(sum, 1, 64);
        if (TPB == 4) sum += __shfl_xor(sum, 2, 64);
        if (part == 0) tot[bin] = sum;
      }
      __syncthreads();
      if (wave == 0) {
        const int b0 = 255 - 4 * lane;          // lane l owns bins 255-4l .. 252-4l, largest digit first
        uint32_t c0 = tot[b0], c1 = tot[b0 - 1], c2 = tot[b0 - 2], c3 = tot[b0 - 3];
        uint32_t sum4 = c0 + c1 + c2 + c3;
        uint32_t incl = sum4;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          uint32_t y = __shfl_up(incl, o, 64);
          if (lane >= o) incl += y;
        }
        uint32_t excl = incl - sum4;
        if (excl < remaining && remaining <= incl) {
          uint32_t r = remaining - excl;
          uint32_t dgt, above;
          if (r <= c0) { dgt = b0; above = excl; }
          else if (r <= c0 + c1) { dgt = b0 - 1; above = excl + c0; }
          else if (r <= c0 + c1 + c2) { dgt = b0 - 2; above = excl + c0 + c1; }
          else { dgt = b0 - 3; above = excl + c0 + c1 + c2; }
          bc[0] = prefix | (dgt << shift);
          bc[1] = remaining - above;
        }
      }
      __syncthreads();
      prefix = bc[0];
      remaining = bc[1];
      mask |= 0xffu << shift;
    }
    tau = prefix;
    need_eq = remaining;
  }

  // ordered compaction over the registers
  uint32_t tot_gt = 0, tot_eq = 0;
#pragma unroll
  for (int j = 0; j < MAXR; ++j) {
    tot_gt += __popcll(__ballot(j < nvalid && k[j] > tau));
    tot_eq += __popcll(__ballot(j < nvalid && k[j] == tau));
  }
  if (lane == 0) { wsum[wave] = tot_gt; wsum[NWAVES + wave] = tot_eq; }
  __syncthreads();
  uint32_t run_gt = 0, run_eq = 0;
  for (int w = 0; w < wave; ++w) { run_gt += wsum[w]; run_eq += wsum[NWAVES + w]; }
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  // kept list: pinned prefix [0, n_pin), then the chosen candidates, then the stabilizers
  int32_t* out = a.kept + (int64_t)m * a.kept_stride + n_pin;
  int32_t* out2 = a.kept2 ? a.kept2 + (int64_t)m * a.stride2 + n_pin : nullptr;
  for (int i = tid; i < n_pin; i += NT) {
    out[i - n_pin] = i;
    if (out2) out2[i - n_pin] = i;
  }
#pragma unroll
  for (int j = 0; j < MAXR; ++j) {
    const bool gt = j < nvalid && k[j] > tau;
    const bool eq = j < nvalid && k[j] == tau;
    const uint64_t bg = __ballot(gt), be = __ballot(eq);
    const uint32_t gt_before = run_gt + __popcll(bg & lt_mask);
    const uint32_t eq_before = run_eq + __popcll(be & lt_mask);
    if (gt || (eq && eq_before < need_eq)) {
      const uint32_t pos = gt_before + min(eq_before, need_eq);
      out[pos] = n_pin + first + j * 64;
      if (out2) out2[pos] = n_pin + first + j * 64;
    }
    run_gt += __popcll(bg);
    run_eq += __popcll(be);
  }
  for (int i = n_cand + tid; i < L - n_pin; i += NT) {
    out[kk + (i - n_cand)] = n_pin + i;
    if (out2) out2[kk + (i - n_cand)] = n_pin + i;
  }
}

constexpr int select_body_smem_words(int nt) { return 256 * SEL_REP + 256 + 2 * (nt / 64) + 2; }

}  // namespace locret
