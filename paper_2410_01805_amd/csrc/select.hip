// Stabilizer-masked top-k per KV head (Section 3.4; Algorithm 1: "+inf on the last n_s, top-b"),
// with an optional pinned prefix (the first n_pin units are kept as well: Locret-Q keeps the query,
// placed at the start of the sequence, visible to every eviction).
//
// One 1024-thread workgroup per KV head.  Scores become order-preserving 32-bit keys (NaN lowest,
// -0 == +0) held in LDS; a 4-pass, 8-bit-per-pass radix select finds the key tau of the k-th best
// candidate and how many units equal to tau still fit; a ballot-based ordered compaction then emits
// the kept indices ascending, taking equal keys from the lowest index up.  Integer work only, so
// the result is exact and deterministic.
//
// Up to 24576 candidates per head the keys never leave registers (select_reg_kernel): wavefront w
// owns a contiguous index range, lane-interleaved in rounds of 64, so every global read is a
// 256-byte line, the radix passes touch LDS only for the histogram, and the final ordered
// compaction is ballots over registers.  Longer inputs use select_kernel (keys in LDS, or re-read
// from global memory when they do not fit).
//
// Histogram counters are replicated 32 times (bin * 32 + lane % 32): every lane of a wavefront then
// updates its own LDS bank whatever digit it holds.  Score keys share their top bits (same sign
// and exponent range), so without the replicas almost all 1024 threads of the first pass would
// queue on two or three counters.
#include "device_util.h"
#include "kernels.h"
#include "select_body.h"

namespace locret {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_HDR = 256 * SEL_REP + 256 + 128;   // words of LDS before the keys: hist[256][32] tot[256] wsum[64] bc[64]

template <bool IN_LDS>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(SelectArgs a) {
  extern __shared__ uint32_t smem[];
  uint32_t* hist = smem;                       // [256][SEL_REP]
  uint32_t* tot = smem + 256 * SEL_REP;        // [256] per-bin totals
  uint32_t* wsum = tot + 256;
  uint32_t* bc = wsum + 64;
  uint32_t* keys = smem + SEL_HDR;

  const int m = blockIdx.x;
  const HeadSel hs = head_sel(a, m);
  const int L = hs.L, n_pin = hs.n_pin;
  int32_t* const kept = a.kept;
  int32_t* const kept2 = a.kept2;
  const int kept_stride = a.kept_stride, stride2 = a.stride2;
  const float* s = a.S + (int64_t)m * a.cap + n_pin;   // candidate c is unit n_pin + c
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int n_cand = L - hs.n_stab - n_pin;
  const int kk = hs.n_keep - hs.n_stab - n_pin;    // candidates to keep, 0 <= kk <= n_cand

  if (IN_LDS)
    for (int i = tid; i < n_cand; i += SEL_THREADS) keys[i] = score_key(s[i]);
  auto key_at = [&](int i) -> uint32_t { return IN_LDS ? keys[i] : score_key(s[i]); };

  uint32_t tau, need_eq;
  if (kk >= n_cand) {          // everything fits
    tau = 0u; need_eq = 0xffffffffu;
    __syncthreads();
  } else if (kk == 0) {        // stabilizers fill the budget
    tau = 0xffffffffu; need_eq = 0u;
    __syncthreads();
  } else {
    uint32_t prefix = 0u, mask = 0u, remaining = (uint32_t)kk;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      for (int i = tid; i < 256 * SEL_REP; i += SEL_THREADS) hist[i] = 0u;
      __syncthreads();
      const int rep = lane & (SEL_REP - 1);
      for (int i = tid; i < n_cand; i += SEL_THREADS) {
        uint32_t key = key_at(i);
        if ((key & mask) == prefix) atomicAdd(&hist[((key >> shift) & 255u) * SEL_REP + rep], 1u);
      }
      __syncthreads();
      {                                        // bin totals: 4 threads per bin, 8 replicas each
        const int bin = tid >> 2, qtr = tid & 3;
        uint32_t sum = 0;
#pragma unroll
        for (int r = 0; r < SEL_REP / 4; ++r) sum += hist[bin * SEL_REP + qtr * (SEL_REP / 4) + r];
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        if (qtr == 0) tot[bin] = sum;
      }
      __syncthreads();
      if (wave == 0) {
        // lane l owns bins 255-4l .. 252-4l; scan from the largest digit down
        const int b0 = 255 - 4 * lane;
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

  // ---- ordered compaction: each wave owns a contiguous range, rounds of 64 consecutive slots ----
  const int wseg = ((n_cand + SEL_WAVES - 1) / SEL_WAVES + 63) & ~63;
  const int w_lo = wave * wseg;
  const int w_hi = min(n_cand, w_lo + wseg);
  uint32_t tot_gt = 0, tot_eq = 0;
  for (int base = w_lo; base < w_hi; base += 64) {
    int i = base + lane;
    uint32_t key = (i < w_hi) ? key_at(i) : 0u;
    bool gt = (i < w_hi) && key > tau;
    bool eq = (i < w_hi) && key == tau;
    tot_gt += __popcll(__ballot(gt));
    tot_eq += __popcll(__ballot(eq));
  }
  if (lane == 0) { wsum[wave] = tot_gt; wsum[SEL_WAVES + wave] = tot_eq; }
  __syncthreads();
  uint32_t run_gt = 0, run_eq = 0;
  for (int w = 0; w < wave; ++w) { run_gt += wsum[w]; run_eq += wsum[SEL_WAVES + w]; }
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  // kept list: pinned prefix [0, n_pin), then the chosen candidates, then the stabilizers
  int32_t* out = kept + (int64_t)m * kept_stride + n_pin;
  int32_t* out2 = kept2 ? kept2 + (int64_t)m * stride2 + n_pin : nullptr;
  for (int i = tid; i < n_pin; i += SEL_THREADS) {
    out[i - n_pin] = i;
    if (out2) out2[i - n_pin] = i;
  }
  for (int base = w_lo; base < w_hi; base += 64) {
    int i = base + lane;
    uint32_t key = (i < w_hi) ? key_at(i) : 0u;
    bool gt = (i < w_hi) && key > tau;
    bool eq = (i < w_hi) && key == tau;
    uint64_t bg = __ballot(gt), be = __ballot(eq);
    uint32_t gt_before = run_gt + __popcll(bg & lt_mask);
    uint32_t eq_before = run_eq + __popcll(be & lt_mask);
    bool keep = gt || (eq && eq_before < need_eq);
    if (keep) {
      uint32_t pos = gt_before + min(eq_before, need_eq);
      out[pos] = n_pin + i;
      if (out2) out2[pos] = n_pin + i;
    }
    run_gt += __popcll(bg);
    run_eq += __popcll(be);
  }
  for (int i = n_cand + tid; i < L - n_pin; i += SEL_THREADS) {
    out[kk + (i - n_cand)] = n_pin + i;
    if (out2) out2[kk + (i - n_cand)] = n_pin + i;
  }
}

// ------------------------------------------------------------------------------------------------
// Register-resident variant: MAXR keys per thread (select_body.h).
template <int MAXR>
__global__ __launch_bounds__(SEL_THREADS) void select_reg_kernel(SelectArgs a) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[select_body_smem_words(SEL_THREADS, 2)];
  select_reg_body<MAXR, SEL_THREADS, 2>(a, blockIdx.x, smem);
}

// bytes of dynamic LDS the in-LDS variant may use: asked for once (thread-safe static initialisation)
static int lds_limit() {
  static const int limit = [] {
    if (hipFuncSetAttribute((const void*)select_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) == hipSuccess)
      return 160 * 1024;
    (void)hipGetLastError();
    return 64 * 1024;
  }();
  return limit;
}

void launch_select(const float* S, int cap, int h_kv, int L, int n_keep, int n_stab, int n_pin, int32_t* kept,
                   int kept_stride, int32_t* kept2, int stride2, hipStream_t st) {
  SelectArgs a = {S, cap, L, n_keep, n_stab, n_pin, kept, kept_stride, kept2, stride2,
                  nullptr, 0, 0, 0, 0, nullptr, nullptr};
  a.L_h.ragged = 0;
  a.keep_h.ragged = 0;
  launch_select(a, h_kv, st);
}

// The path is chosen for the longest head; every path takes shorter heads as they come.
void launch_select(const SelectArgs& a, int h_kv, hipStream_t st) {
  const int ns = a.n_stab < a.L ? a.n_stab : a.L;
  const int npin = a.n_pin < a.L - ns ? a.n_pin : a.L - ns;
  const int n_cand = a.L - ns - npin;
  const int wseg = ((n_cand + SEL_WAVES - 1) / SEL_WAVES + 63) & ~63;
  if (wseg <= 12 * 64) {
    launch_kernel(select_reg_kernel<12>, dim3(h_kv), dim3(SEL_THREADS), 0, st, a);
    return;
  }
  if (wseg <= 24 * 64) {
    launch_kernel(select_reg_kernel<24>, dim3(h_kv), dim3(SEL_THREADS), 0, st, a);
    return;
  }
  size_t need = (size_t)(SEL_HDR + n_cand) * sizeof(uint32_t);
  if (need <= (size_t)lds_limit())
    launch_kernel(select_kernel<true>, dim3(h_kv), dim3(SEL_THREADS), need, st, a);
  else
    launch_kernel(select_kernel<false>, dim3(h_kv), dim3(SEL_THREADS), SEL_HDR * sizeof(uint32_t), st, a);
}

}  // namespace locret
