// Chunk attention (Eq. 1) on the bf16 matrix cores of gfx950, software-pipelined variant.
//
// Same data flow as attention_bf16.hip (transposed products S^T = K Q^T and O^T += V^T P^T with
// v_mfma_f32_32x32x16_bf16, K tile [64][D+8] and transposed V tile [D][64+8] in LDS, buffer-load
// staging), but the online softmax advances in HALF tiles of 32 keys and the matrix and vector
// pipes are kept busy at the same time inside every wavefront:
//
//   sub-step h:   MFMA  S(h+1) = K_half(h+1) Q^T          |  VALU  P(h) = exp2(S(h) c - m c), row sums
//                 MFMA  O^T   += V^T_half(h) P(h)^T       |  VALU  row max of S(h+1), staging transposes
//
// S(h+1) is produced one sub-step ahead of its use, so the exponentials of half h never wait for a
// matrix product; the running max that half h+1 will be scaled by is settled between sub-steps
// (a rarely taken branch: the max is only raised when a probability would exceed 2^8, and O and l
// are rescaled then).  Each sub-step is one straight-line block whose issue order is pinned with
// scheduling-group barriers: one MFMA, one LDS fragment read for a later MFMA, a handful of VALU
// instructions, repeated.
//
// LDS hand-over with one barrier per sub-step: K tile i is read in sub-steps 2i-1 and 2i, V tile i
// in sub-steps 2i and 2i+1.  K tile i+1 is written during sub-step 2i and V tile i+1 during
// sub-step 2i+1, each into the buffer whose last reader finished two barriers earlier; the global
// loads that feed them are issued two sub-steps before.
#include "attn_common.h"
#include "kernels.h"

namespace locret {

template <int D>
__global__ __launch_bounds__(256, 2) void attn_pipe_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kx,
                                                           const bf16_t* __restrict__ V, bf16_t* __restrict__ out,
                                                           int Tn, int h, int g, int cap, int n_c_common, float c_log2,
                                                           int hpw, int n_hgroups, int n_ttiles, HeadLens n_c_h) {
  constexpr int NKS = D / 16;          // k-steps over the head dim for S
  constexpr int NDB = D / 32;          // 32-row blocks of O^T
  constexpr int KCH = D / 8;           // 16-byte chunks per K row
  constexpr int K_LD = (KT * KCH) / 256;   // K chunks per thread per tile
  constexpr int V_BLK = (KT / 4) * KCH;    // 4-key x 8-dim blocks per V tile
  constexpr int KSTR = AttnSmem<D>::KSTR;
  constexpr int VSTR = AttnSmem<D>::VSTR;
  __shared__ AttnSmem<D> sm;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: everything derived from it is wave-uniform
  const int n32 = lane & 31;
  const int hi = lane >> 5;

  // ---- workgroup -> (head group, token tile): one KV head per XCD, longest key ranges first -----
  const int bid = blockIdx.x;
  int hgroup, tt;
  if ((n_hgroups & 7) == 0) {
    const int g8 = n_hgroups >> 3;
    hgroup = (bid & 7) * g8 + (bid >> 3) % g8;
    tt = bid / n_hgroups;
  } else {
    hgroup = bid % n_hgroups;
    tt = bid / n_hgroups;
  }
  tt = n_ttiles - 1 - tt;
  const int wph = 4 / hpw;                     // wavefronts per head
  const int TW = wph * 32;                     // tokens per workgroup
  const int t0 = tt * TW;
  const int j = hgroup * hpw + wave / wph;     // query head of this wavefront
  const int m = (hgroup * hpw) / g;            // KV head: the same for all four wavefronts
  const int n_c = __builtin_amdgcn_readfirstlane(head_len(n_c_h, m, n_c_common));   // this KV head's cache length
  const int tw0 = t0 + (wave % wph) * 32;      // first token of this wavefront
  const int t_last_wg = min(Tn, t0 + TW) - 1;
  const int n_keys = n_c + t_last_wg + 1;      // slots the workgroup stages
  const int n_tiles = (n_keys + KT - 1) / KT;
  const int my_t = min(tw0 + n32, Tn - 1);     // this lane's query token (clamped: extra rows are discarded)
  const int limit = n_c + my_t;                // last slot this lane's query sees
  const int tw0c = min(tw0, Tn - 1);
  const int wave_last_half = (n_c + min(Tn - 1, tw0 + 31)) >> 5;   // last 32-key half any lane of the wave sees
  const int first_mask_half = (n_c + tw0c + 1) >> 5;               // halves from here on may cross the diagonal

  // per-head bases, forced into scalar registers (the 64-bit multiply is done on the vector unit)
  auto scalar_ptr = [](const bf16_t* p) -> const bf16_t* {
    uint64_t a = (uint64_t)p;
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    uint32_t hi32 = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return (const bf16_t*)(((uint64_t)hi32 << 32) | lo);
  };
  const bf16_t* Kb = scalar_ptr(Kx + (int64_t)m * cap * D);
  const bf16_t* Vb = scalar_ptr(V + (int64_t)m * cap * D);

  bf16x8 qf[NKS];
  {
    const bf16_t* qp = q + ((int64_t)my_t * h + j) * D + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const bf16x8*)(qp + ks * 16);
  }
  f32x16 oacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run, l_run = 0.f;

  // ---- staging (see attention_bf16.hip): buffer loads zero-fill past the staged slots ------------
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  uint4 kreg[K_LD];
  uint4 vreg[4];
  const int v_id = (V_BLK == 256) ? tid : (tid >= V_BLK ? tid - V_BLK : tid);   // spare threads repeat a block
  const int v_kq = v_id & 15;
  const int v_d8 = v_id >> 4;
  // chunk tid + 256 i of a K tile: global byte offset (tid + 256 i) * 16 (the i part goes into the
  // buffer descriptor), LDS element offset row * KSTR + col * 8
  constexpr bool K_POW2 = (KCH & (KCH - 1)) == 0;
  const int k_go = tid * 16;
  int k_st[K_LD];
#pragma unroll
  for (int i = 0; i < K_LD; ++i) {
    int c = tid + 256 * i;
    k_st[i] = K_POW2 ? ((tid / KCH) * KSTR + (tid % KCH) * 8 + i * (256 / KCH) * KSTR) : ((c / KCH) * KSTR + (c % KCH) * 8);
  }
  const int v_go = ((v_kq * 4) * D + v_d8 * 8) * 2;
  const int v_qg = v_kq & 3;
  const int v_kqp = (v_kq & ~3) | ((v_qg == 1) ? 2 : (v_qg == 2) ? 1 : v_qg);   // keys of 16 as 0-3, 8-11, 4-7, 12-15
  const int v_st = (v_d8 * 8) * VSTR + v_kqp * 4;
  const int k_rd = n32 * KSTR + hi * 8;
  const int v_rd = n32 * VSTR + hi * 8;

  // descriptors are built from wave-uniform values only (kept in scalar registers)
  auto load_K = [&](int tile) {
    const int tile_u = __builtin_amdgcn_readfirstlane(tile);
    const int left = max(n_keys - tile_u * KT, 0) * (D * 2);
#pragma unroll
    for (int i = 0; i < K_LD; ++i) {
      __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(Kb + (int64_t)tile_u * (KT * D) + i * 2048), 0,
          __builtin_amdgcn_readfirstlane(max(left - i * 4096, 0)), 0x00020000);
      u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(kr, k_go, 0, 0);
      kreg[i] = make_uint4(x[0], x[1], x[2], x[3]);
    }
  };
  auto load_V = [&](int tile) {
    const int tile_u = __builtin_amdgcn_readfirstlane(tile);
    const int left = __builtin_amdgcn_readfirstlane(max(n_keys - tile_u * KT, 0) * (D * 2));
    __amdgpu_buffer_rsrc_t vr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Vb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(vr, v_go + i * (D * 2), 0, 0);
      vreg[i] = make_uint4(x[0], x[1], x[2], x[3]);
    }
  };
  auto store_K = [&](int buf) {
    bf16_t* dst = sm.K[buf];
#pragma unroll
    for (int i = 0; i < K_LD; ++i) *(uint4*)(dst + k_st[i]) = kreg[i];
  };
  auto store_V = [&](int buf) {
    bf16_t* dst = sm.Vt[buf] + v_st;
    const uint32_t* r0 = (const uint32_t*)&vreg[0];
    const uint32_t* r1 = (const uint32_t*)&vreg[1];
    const uint32_t* r2 = (const uint32_t*)&vreg[2];
    const uint32_t* r3 = (const uint32_t*)&vreg[3];
#pragma unroll
    for (int p = 0; p < 4; ++p) {              // word p holds dims 2p (low half) and 2p+1 (high half)
      uint2 even, odd;
      even.x = (r0[p] & 0xffffu) | (r1[p] << 16);
      even.y = (r2[p] & 0xffffu) | (r3[p] << 16);
      odd.x = (r0[p] >> 16) | (r1[p] & 0xffff0000u);
      odd.y = (r2[p] >> 16) | (r3[p] & 0xffff0000u);
      *(uint2*)(dst + (2 * p) * VSTR) = even;
      *(uint2*)(dst + (2 * p + 1) * VSTR) = odd;
    }
  };
  // Staging work of one sub-step: even sub-steps hand over K of the next tile, odd ones V, and
  // start the loads of the tile after it.  Unconditional: past the last tile the loads return
  // zeros without touching memory and the stores land in a buffer nobody reads again.
  auto stage = [&](auto parc, int tile) {
    constexpr int PAR = decltype(parc)::value;
    if constexpr (PAR == 0) {
      store_K((tile + 1) & 1);
      load_K(tile + 2);
    } else {
      store_V((tile + 1) & 1);
      load_V(tile + 2);
    }
  };

  // mask (if the half may cross the diagonal) and row max of a freshly computed S half
  auto mask_and_max = [&](f32x16& s, int half, bool mask) -> float {
    if (mask) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int slot = half * 32 + (r >> 2) * 8 + hi * 4 + (r & 3);
        if (slot > limit) s[r] = -INFINITY;
      }
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    return max_across_halves(mx);
  };

  f32x16 s_a, s_b;            // S halves: one being consumed, one being produced (roles alternate)
  float mx_nxt;

  // ---- one sub-step as a single scheduled block --------------------------------------------------
  auto compute = [&](auto parc, auto maskc, int hh, const f32x16& s_cur, f32x16& s_nxt) {
    constexpr int PAR = decltype(parc)::value;
    constexpr bool MASK = decltype(maskc)::value;
    const int tile = hh >> 1;
    const bf16_t* Kn = sm.K[(tile + PAR) & 1] + k_rd + (1 - PAR) * 32 * KSTR;   // half hh+1
    const bf16_t* Vc = sm.Vt[tile & 1] + v_rd + PAR * 32;                       // half hh: keys PAR*32 ..
    bf16x8 kf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) kf[ks] = *(const bf16x8*)(Kn + ks * 16);
    bf16x8 vf[2][NDB];
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
      for (int db = 0; db < NDB; ++db) vf[kc][db] = *(const bf16x8*)(Vc + db * 32 * VSTR + kc * 16);
    // S(hh+1)
#pragma unroll
    for (int r = 0; r < 16; ++r) s_nxt[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s_nxt, 0, 0, 0);
    // P(hh)
    const float mc = m_run * c_log2;
    float p[16];
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      p[r] = __builtin_amdgcn_exp2f(fmaf(s_cur[r], c_log2, -mc));
      psum += p[r];
    }
    l_run += psum;
    uint4 pb[2];
    pb[0] = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
    pb[1] = make_uint4(pack_bf16(p[8], p[9]), pack_bf16(p[10], p[11]), pack_bf16(p[12], p[13]), pack_bf16(p[14], p[15]));
    // O^T += V^T P^T
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
      for (int db = 0; db < NDB; ++db)
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kc][db], *(const bf16x8*)&pb[kc], oacc[db], 0, 0, 0);
    mx_nxt = mask_and_max(s_nxt, hh + 1, MASK);
    stage(parc, tile);

    // issue order: 4 fragment reads ahead, then MFMA / LDS read / VALU interleaved
    constexpr int N_RD = NKS + 2 * NDB;
    constexpr int AHEAD = 4;
    constexpr int V1 = (64 + NKS - 1) / NKS;
    __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
    for (int i = 0; i < NKS; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, V1, 0);
    }
    if constexpr (N_RD - AHEAD - NKS > 0) __builtin_amdgcn_sched_group_barrier(0x100, N_RD - AHEAD - NKS, 0);
#pragma unroll
    for (int i = 0; i < 2 * NDB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, MASK ? 10 : 6, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x200, PAR == 0 ? K_LD : 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x020, PAR == 0 ? K_LD : 4, 0);
  };

  // settle the max the next half is scaled by (between sub-steps, after the barrier)
  auto settle = [&](int hh) {
    if (hh + 1 <= wave_last_half) {
      const float m_new = fmaxf(m_run, mx_nxt);
      if (__any((m_new - m_run) * c_log2 > RESCALE_LOG2)) {
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
      }
    }
  };

  // ---- prologue: tile 0 in LDS, tile 1 in flight, S(0) and its max ---------------------------------
  load_K(0);
  load_V(0);
  store_K(0);
  load_K(1);
  store_V(0);
  load_V(1);
  __syncthreads();
  {
    f32x16& s_nxt = s_a;
#pragma unroll
    for (int r = 0; r < 16; ++r) s_nxt[r] = 0.f;
    const bf16_t* K0 = sm.K[0] + k_rd;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
      s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(K0 + ks * 16), qf[ks], s_nxt, 0, 0, 0);
    m_run = mask_and_max(s_nxt, 0, true);      // finite: slot 0 is visible to every query
  }

  // Tiles whose halves all lie left of this wavefront's diagonal run unmasked; the rest apply the
  // causal mask and let wavefronts that have run out of visible keys only stage and synchronise.
  // Every wavefront executes 2 * n_tiles barriers in total.
  const int t_plain = min(n_tiles, max(0, (first_mask_half - 1) >> 1));
  int tile = 0;
  for (; tile < t_plain; ++tile) {
    compute(IntC<0>(), IntC<0>(), 2 * tile, s_a, s_b);
    __syncthreads();
    settle(2 * tile);
    compute(IntC<1>(), IntC<0>(), 2 * tile + 1, s_b, s_a);
    __syncthreads();
    settle(2 * tile + 1);
  }
  for (; tile < n_tiles; ++tile) {
    if (2 * tile <= wave_last_half) compute(IntC<0>(), IntC<1>(), 2 * tile, s_a, s_b);
    else stage(IntC<0>(), tile);
    __syncthreads();
    settle(2 * tile);
    if (2 * tile + 1 <= wave_last_half) compute(IntC<1>(), IntC<1>(), 2 * tile + 1, s_b, s_a);
    else stage(IntC<1>(), tile);
    __syncthreads();
    settle(2 * tile + 1);
  }

  // ---- epilogue: O = O^T / l; lane holds 4 consecutive dims per (db, r/4) for its query -------------
  {
    const int t = tw0 + n32;
    float l = l_run + __shfl_xor(l_run, 32, 64);
    if (t < Tn) {
      const float inv = 1.f / l;
      bf16_t* op = out + ((int64_t)t * h + j) * D;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          uint2 w;
          w.x = pack_bf16(oacc[db][rq * 4 + 0] * inv, oacc[db][rq * 4 + 1] * inv);
          w.y = pack_bf16(oacc[db][rq * 4 + 2] * inv, oacc[db][rq * 4 + 3] * inv);
          *(uint2*)(op + db * 32 + rq * 8 + hi * 4) = w;
        }
    }
  }
}

template <int D>
static void pipe_launch(const Dims& Dm, const void* q, const void* Kx, const void* V, void* out, int T, int n_c,
                        float scale, hipStream_t st, const HeadLens& hl) {
  const int g = Dm.g;
  const int hpw = (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
  const int wph = 4 / hpw;
  const int TW = wph * 32;
  const int n_hgroups = Dm.h / hpw;
  const int n_ttiles = (T + TW - 1) / TW;
  const float c_log2 = scale * 1.4426950408889634f;
  hipLaunchKernelGGL((attn_pipe_kernel<D>), dim3(n_hgroups * n_ttiles), dim3(256), 0, st, (const bf16_t*)q,
                     (const bf16_t*)Kx, (const bf16_t*)V, (bf16_t*)out, T, Dm.h, g, Dm.cap, n_c, c_log2, hpw,
                     n_hgroups, n_ttiles, hl);
}

bool launch_attention_bf16_pipe(const Dims& Dm, const void* q, const void* Kx, const void* V, void* out, int T,
                                int n_c, float scale, hipStream_t st, const HeadLens* n_c_h) {
  const HeadLens hl = head_lens_or_common(n_c_h);
  switch (Dm.d) {
    case 64: pipe_launch<64>(Dm, q, Kx, V, out, T, n_c, scale, st, hl); return true;
    case 96: pipe_launch<96>(Dm, q, Kx, V, out, T, n_c, scale, st, hl); return true;
    case 128: pipe_launch<128>(Dm, q, Kx, V, out, T, n_c, scale, st, hl); return true;
    default: return false;
  }
}

}  // namespace locret
