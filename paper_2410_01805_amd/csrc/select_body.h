// Exact top-k selection over the retaining-head scores of one KV head with the keys held in registers
// (the body of select_reg_kernel, also run by workgroups of the head_dim-128 attention launch): see
// select.hip for the method.  NT threads (512 or 1024), MAXR keys per thread, MAXR * 64 * (NT / 64) >= the
// number of candidates.  smem: select_body_smem_words(NT, REP1) words.
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

constexpr int SEL_REP = 32;    // counter replicas per bin of the 8-bit passes of select_kernel (= LDS banks)

// Digits of the register-resident form: 12 + 10 + 10 bits, most significant first.  Score keys share their sign
// and most exponent bits, so an 8-bit first digit leaves a third of the candidates in the threshold's bin and
// the second pass as heavy as the first; a 12-bit one (sign, exponent, 3 mantissa bits) leaves a few percent,
// and the two remaining passes see almost no key: three passes, of which one costs.
constexpr int SEL_BITS1 = 12, SEL_BITS2 = 10;
constexpr int SEL_NB1 = 1 << SEL_BITS1, SEL_NB2 = 1 << SEL_BITS2;
constexpr int SEL_REP2 = 2;    // replicas per bin of the two 10-bit passes (they see few keys)

// sum of ws[0 .. wave) for NWAVES <= 16 words of LDS: every thread reads all of them with 16-byte loads (one
// latency) instead of walking them one by one
template <int NWAVES>
__device__ __forceinline__ uint32_t sum_before(const uint32_t* ws, int wave) {
  static_assert(NWAVES % 4 == 0 && NWAVES <= 16, "wave totals as 16-byte vectors");
  uint32_t acc = 0;
#pragma unroll
  for (int q = 0; q < NWAVES / 4; ++q) {
    const uint4 v = *(const uint4*)(ws + 4 * q);
    acc += (4 * q + 0 < wave ? v.x : 0u) + (4 * q + 1 < wave ? v.y : 0u) + (4 * q + 2 < wave ? v.z : 0u) +
           (4 * q + 3 < wave ? v.w : 0u);
  }
  return acc;
}

// One radix pass over the keys k[0 .. nvalid) of every thread that still match `prefix` under `mask`: counts the
// digit (k >> shift) & (NB - 1) in hist[NB][REP] (zero on entry), finds from the top the digit that holds the
// remaining-th key and updates prefix / remaining.  Returns true when every key of that digit is wanted (the digit
// holds exactly `remaining` keys): the lower bits then need no pass.  All NT threads call it; scratch: ws[16 + 3],
// 16-byte aligned, private to the pass.
template <int MAXR, int NT, int NB, int REP>
__device__ __forceinline__ bool select_radix_pass(const uint32_t (&k)[MAXR], int nvalid, int shift, uint32_t mask,
                                                  uint32_t& prefix, uint32_t& remaining, uint32_t* hist, uint32_t* ws) {
  constexpr int NWAVES = NT / 64;
  constexpr int BPT = NB / NT;                 // bins per thread in the scan
  static_assert(NB % NT == 0 && BPT >= 1, "bins per thread");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = lane & (REP - 1);
#pragma unroll
  for (int j = 0; j < MAXR; ++j)
    if (j < nvalid && (k[j] & mask) == prefix) atomicAdd(&hist[((k[j] >> shift) & (uint32_t)(NB - 1)) * REP + rep], 1u);
  __syncthreads();
  // thread t owns bins NB-1 - t BPT - i, i < BPT: ascending thread order = descending digits
  uint32_t c[BPT];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    const int bin = NB - 1 - tid * BPT - i;
    uint32_t x = 0;
#pragma unroll
    for (int r = 0; r < REP; ++r) x += hist[bin * REP + r];
    c[i] = x;
    sum += x;
  }
  uint32_t incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(incl, o, 64);
    if (lane >= o) incl += y;
  }
  if (lane == 63) ws[wave] = incl;
  __syncthreads();
  const uint32_t excl = sum_before<NWAVES>(ws, wave) + incl - sum;
  if (excl < remaining && remaining <= excl + sum) {      // exactly one thread
    uint32_t above = excl;
    int i = 0;
#pragma unroll
    for (int u = 0; u < BPT - 1; ++u)
      if (i == u && remaining > above + c[u]) { above += c[u]; i = u + 1; }
    const uint32_t dgt = (uint32_t)(NB - 1 - tid * BPT - i);
    uint32_t cnt = c[0];
#pragma unroll
    for (int u = 1; u < BPT; ++u) cnt = (i == u) ? c[u] : cnt;
    ws[16] = prefix | (dgt << shift);
    ws[17] = remaining - above;
    ws[18] = cnt;
  }
  __syncthreads();
  prefix = ws[16];
  remaining = ws[17];
  return remaining == ws[18];
}

// REP1: replicas per bin of the first pass (4 where 64 KB of LDS are at hand, else 2)
template <int MAXR, int NT, int REP1>
__device__ __forceinline__ void select_reg_body(const SelectArgs& a, int m, uint32_t* smem) {
  static_assert(NT == 512 || NT == 1024, "workgroup sizes of the two callers");
  constexpr int NWAVES = NT / 64;
  // a histogram per pass, all cleared at once beside the loads of the keys: [bins][replicas]
  constexpr int H1 = SEL_NB1 * REP1, H2 = SEL_NB2 * SEL_REP2;
  uint32_t* hist = smem;                       // pass 1, then pass 2 at + H1, pass 3 at + H1 + H2
  uint32_t* ws = hist + H1 + 2 * H2;           // [3][20] scan scratch of the passes (16-byte aligned)
  uint32_t* wsum = ws + 3 * 20;                // [2][16] totals per wavefront of the emit
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
    for (int i = tid; i < (H1 + 2 * H2) / 4; i += NT) ((uint4*)hist)[i] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < MAXR; ++j) k[j] = score_key(f[j]);
  }

  uint32_t tau, need_eq;
  if (kk >= n_cand) {
    tau = 0u; need_eq = 0xffffffffu;
  } else if (kk == 0) {
    tau = 0xffffffffu; need_eq = 0u;
  } else {
    uint32_t prefix = 0u, remaining = (uint32_t)kk;
    // A pass may end the search early: when the digit it settles on holds exactly the keys still wanted, all
    // keys with that prefix are kept, whatever their lower bits: tau = the prefix with zeros below, every key equal
    // to it kept.  (After the second pass the digit typically holds one key.)
    bool all = select_radix_pass<MAXR, NT, SEL_NB1, REP1>(k, nvalid, 32 - SEL_BITS1, 0u, prefix, remaining, hist, ws);
    if (!all) all = select_radix_pass<MAXR, NT, SEL_NB2, SEL_REP2>(k, nvalid, SEL_BITS2, ~0u << (32 - SEL_BITS1), prefix, remaining, hist + H1, ws + 20);
    if (!all) all = select_radix_pass<MAXR, NT, SEL_NB2, SEL_REP2>(k, nvalid, 0, ~0u << SEL_BITS2, prefix, remaining, hist + H1 + H2, ws + 40);
    tau = prefix;
    need_eq = remaining;
  }

  // ---- ordered compaction over the registers ---------------------------------------------------------------
  // totals per wavefront: kept-for-sure keys (> tau) by ballots, keys equal to tau counted per thread first
  uint32_t tot_gt = 0, my_eq = 0;
#pragma unroll
  for (int j = 0; j < MAXR; ++j) {
    tot_gt += __popcll(__ballot(j < nvalid && k[j] > tau));
    my_eq += (j < nvalid && k[j] == tau) ? 1u : 0u;
  }
  uint32_t tot_eq = my_eq;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) tot_eq += __shfl_xor(tot_eq, o, 64);
  if (lane == 0) { wsum[wave] = tot_gt; wsum[16 + wave] = tot_eq; }
  __syncthreads();
  uint32_t run_gt = sum_before<NWAVES>(wsum, wave), run_eq = sum_before<NWAVES>(wsum + 16, wave);
  // kept list: pinned prefix [0, n_pin), then the chosen candidates, then the stabilizers
  int32_t* out = a.kept + (int64_t)m * a.kept_stride + n_pin;
  int32_t* out2 = a.kept2 ? a.kept2 + (int64_t)m * a.stride2 + n_pin : nullptr;
  for (int i = tid; i < n_pin; i += NT) {
    out[i - n_pin] = i;
    if (out2) out2[i - n_pin] = i;
  }
  if (tot_eq == 0) {
    // the common case, decided per wavefront: none of its keys equals tau, so a key is kept iff it is above tau and
    // its place is the count of kept keys before it (the equal keys of earlier wavefronts add a constant)
    uint32_t base = run_gt + min(run_eq, need_eq);
#pragma unroll
    for (int j = 0; j < MAXR; ++j) {
      const bool gt = j < nvalid && k[j] > tau;
      const uint64_t bg = __ballot(gt);
      if (gt) {
        const uint32_t pos = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(bg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bg, 0u));
        out[pos] = n_pin + first + j * 64;
        if (out2) out2[pos] = n_pin + first + j * 64;
      }
      base += __popcll(bg);
    }
  } else {
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
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
  }
  for (int i = n_cand + tid; i < L - n_pin; i += NT) {
    out[kk + (i - n_cand)] = n_pin + i;
    if (out2) out2[kk + (i - n_cand)] = n_pin + i;
  }
}

constexpr int select_body_smem_words(int nt, int rep1) { return SEL_NB1 * rep1 + 2 * SEL_NB2 * SEL_REP2 + 3 * 20 + 2 * 16; }

}  // namespace locret
