// Chunk attention (Eq. 1) on the bf16 matrix cores of gfx950.
//
// For each query head j (KV head m = j / g) and query token t of the chunk, keys are the slots
// [0, n_c + t] of one contiguous K/V array per KV head (retained cache followed by the chunk);
// softmax is computed online in fp32.
//
// Workgroup = 4 wavefronts.  Each wavefront owns QB blocks of 32 queries of one head; the
// wavefronts of a workgroup share one KV head, so the K/V tiles they stage in LDS are read by
// every one of them (for g >= 4 the four wavefronts are four query heads of the same group over
// the same tokens; for g = 1 they are four token ranges of one head).
//
// The products are formed transposed, with v_mfma_f32_32x32x16_bf16:
//   S^T[key][query] = K[key][:] . Q[query][:]      A = K tile rows (LDS), B = Q (registers)
//   O^T[dim][query] += V^T[dim][key] . P^T[key][query]   A = V^T (LDS), B = P^T (registers)
// In the 32x32 accumulator layout a lane holds, for ONE query (column lane%32), 16 keys of a
// 32-key block: keys (r/4)*8 + (lane/32)*4 + r%4 for register r.  Hence the running max, the
// rescale factor and the row sum are per-lane scalars, the only cross-lane step being one
// exchange with lane^32, and P^T leaves the accumulator already in B-operand order provided the
// V^T tile stores its keys in the matching order (each group of 16 keys as 0-3, 8-11, 4-7, 12-15).
//
// Softmax as in attention_pp.hip: queries pre-scaled by scale * log2(e) (and rotated here when the
// rotary table is passed), S chains started from -(running max), exp2 / bf16 pack / two-way dot
// products per tile, the running max moved only on the first tile and when a lane's probability
// sum reaches 2^30.
//
// K tile in LDS: [64 keys][D + 8]; V^T tile in LDS: [D][64 + 8], transposed on the way in by 4x8
// register blocks.  The 16-byte row pad makes the stride an odd number of 16-byte chunks, so the
// 16-byte row reads of consecutive lanes and the 8-byte transposing writes both spread over all
// banks, and every LDS address is "per-thread base + compile-time offset".  Tiles are double
// buffered through registers (one barrier per 64 keys); the tile loop is unrolled by two so the
// buffer index is a compile-time constant, and only the last tile pays for bounds checks.
#include <hip/hip_ext.h>
#include <string.h>

#include "attn_common.h"
#include "kernels.h"

namespace locret {

template <int D, int QB, int NW, int WPE>
__global__ __launch_bounds__(NW * 64, WPE) void attn_mfma_kernel(const bf16_t* __restrict__ q, const float2* __restrict__ tab,
                                                             const bf16_t* __restrict__ Kx, const bf16_t* __restrict__ V,
                                                             bf16_t* __restrict__ out,
                                                             int Tn, int h, int g, int cap, int n_c_common, float c_log2,
                                                             int hpw, int n_hgroups, int n_ttiles, HeadLens n_c_h,
                                                             int spread, HeadOrder order) {
  constexpr int NKS = D / 16;          // k-steps over the head dim for S
  constexpr int NDB = D / 32;          // 32-row blocks of O^T
  constexpr int KCH = D / 8;           // 16-byte chunks per K row
  constexpr int K_LD = (KT * KCH) / 256;   // K chunks per staging thread per tile
  constexpr int V_BLK = (KT / 4) * KCH;    // 4-key x 8-dim blocks per V tile
  constexpr int KSTR = AttnSmem<D>::KSTR;
  constexpr int VSTR = AttnSmem<D>::VSTR;
  __shared__ AttnSmem<D> sm;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: everything derived from it is wave-uniform
  const int n32 = lane & 31;
  const int hi = lane >> 5;

  // ---- workgroup -> (head group, token tile); consecutive ids go to different XCDs, so the
  // ---- head group is taken from id % 8 to keep one KV head's K/V in one XCD's L2 --------------
  const int bid = blockIdx.x;
  int hgroup, tt;
  if (spread) {
    // KV heads of different cache lengths (head-wise budgets): every XCD takes every eighth token tile of
    // every head, longest head first, so that no XCD is left with the long heads (see attention_pp.hip)
    const int i = bid >> 3, per_head = (n_ttiles + 7) >> 3;
    const int r = i / per_head;
    const int gph = g / hpw;                               // head groups per KV head
    hgroup = order.v[r / gph] * gph + r % gph;
    tt = (i % per_head) * 8 + (bid & 7);
    if (tt >= n_ttiles) return;                            // the launch is padded to whole rounds of the 8 XCDs
  } else if ((n_hgroups & 7) == 0) {
    const int g8 = n_hgroups >> 3;
    hgroup = (bid & 7) * g8 + (bid >> 3) % g8;
    tt = bid / n_hgroups;
  } else {
    hgroup = bid % n_hgroups;
    tt = bid / n_hgroups;
  }
  tt = n_ttiles - 1 - tt;                      // longest key ranges first
  const int wph = NW / hpw;                    // wavefronts per head
  const int TW = wph * 32 * QB;                // tokens per workgroup
  const int t0 = tt * TW;
  const int j = hgroup * hpw + wave / wph;     // query head of this wavefront
  const int m = (hgroup * hpw) / g;            // KV head: the same for all four wavefronts (blockIdx only)
  const int n_c = __builtin_amdgcn_readfirstlane(head_len(n_c_h, m, n_c_common));   // this head's cache length
  const int tw0 = t0 + (wave % wph) * 32 * QB; // first token of this wavefront
  const int t_last_wg = min(Tn, t0 + TW) - 1;
  const int n_keys = n_c + t_last_wg + 1;      // slots the workgroup stages
  const int n_tiles = (n_keys + KT - 1) / KT;
  const int wave_last_slot = n_c + min(Tn - 1, tw0 + 32 * QB - 1);

  const bf16_t* Kb = Kx + (int64_t)m * cap * D;
  const bf16_t* Vb = V + (int64_t)m * cap * D;

  // ---- Q fragments: B operand, lane = query n32 of block qb, dims ks*16 + hi*8 .. +8 ------------
  bf16x8 qf[QB][NKS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int t = min(tw0 + qb * 32 + n32, Tn - 1);
    const bf16_t* qp = q + ((int64_t)t * h + j) * D + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[qb][ks] = *(const bf16x8*)(qp + ks * 16);
    // Queries are scaled by scale * log2(e) here, so logits leave the MFMA in log2 units; with `tab`
    // they arrive un-rotated and are rotated to position n_c + t first (pairs (i, i + D/2) sit in
    // fragments ks and ks + NKS/2 of the same lane).  One rounding to bf16 either way.
    if (tab != nullptr) {
      const float2* tp = tab + (int64_t)(n_c + t) * (D / 2) + hi * 8;
#pragma unroll
      for (int ks = 0; ks < NKS / 2; ++ks) {
        float lo[8], up[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float2 cs = tp[ks * 16 + e];
          const float a = (float)qf[qb][ks][e], b = (float)qf[qb][ks + NKS / 2][e];
          lo[e] = (a * cs.x - b * cs.y) * c_log2;
          up[e] = (b * cs.x + a * cs.y) * c_log2;
        }
        uint4 pl = make_uint4(pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]), pack_bf16(lo[4], lo[5]), pack_bf16(lo[6], lo[7]));
        uint4 pu = make_uint4(pack_bf16(up[0], up[1]), pack_bf16(up[2], up[3]), pack_bf16(up[4], up[5]), pack_bf16(up[6], up[7]));
        qf[qb][ks] = __builtin_bit_cast(bf16x8, pl);
        qf[qb][ks + NKS / 2] = __builtin_bit_cast(bf16x8, pu);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (float)qf[qb][ks][e] * c_log2;
        uint4 px = make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
        qf[qb][ks] = __builtin_bit_cast(bf16x8, px);
      }
    }
  }

  f32x16 oacc[NDB][QB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
  // Softmax state per query block: running max m_run (log2 units), running sum l_run, and negm = -m_run
  // in all 16 registers: every S chain starts from it, so the MFMA result is (logit - running max) and
  // exp2 applies to it directly.  `fresh` (wave-uniform) is true until the first tile has set the max.
  float m_run[QB], l_run[QB];
  f32x16 negm[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = 0.f;
    l_run[qb] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[qb][r] = 0.f;
  }
  bool fresh = true;

  // ---- staging: a K tile is one contiguous block of KT*KCH 16-byte chunks, 256 threads take
  // ---- chunks st + 256 i; a V tile is cut into 4-key x 8-dim blocks, one per thread of 256.
  // ---- With 4 wavefronts every thread does both; with 8, wavefronts 0-3 stage V and 4-7 stage K
  // ---- (one register set serves either role).
  constexpr bool SPLIT = NW == 8;
  const bool do_k = !SPLIT || wave >= 4;
  const bool do_v = !SPLIT || wave < 4;
  const int st = tid & 255;
  uint4 kreg[4];
  uint4 vreg_own[SPLIT ? 1 : 4];
  uint4* vreg = SPLIT ? kreg : vreg_own;
  const int v_kq = st & 15;                    // key quad: fastest over lanes -> contiguous LDS writes
  const int v_d8 = st >> 4;                    // 8-dim column group
  const bool v_on = do_v && st < V_BLK;
  // Tiles are fetched with buffer loads whose descriptor covers exactly the slots this
  // workgroup may stage: a read past them returns zero, so the last (partial) tile needs no
  // branch and no load ever waits on a predicate.
  int k_go[K_LD];                              // byte offset of chunk tid + 256 i inside a K tile
#pragma unroll
  for (int i = 0; i < K_LD; ++i) k_go[i] = (st + 256 * i) * 16;
  const int v_go = ((v_kq * 4) * D + v_d8 * 8) * 2;                      // + i*D*2
  int k_st[K_LD];                              // LDS element offset of each staged K chunk
#pragma unroll
  for (int i = 0; i < K_LD; ++i) {
    int c = st + 256 * i;
    k_st[i] = (c / KCH) * KSTR + (c % KCH) * 8;
  }
  // V^T destination of this thread's block: rows v_d8*8 + e, key-quad position with the keys of
  // each group of 16 stored as 0-3, 8-11, 4-7, 12-15
  const int v_qg = v_kq & 3;
  const int v_kqp = (v_kq & ~3) | ((v_qg == 1) ? 2 : (v_qg == 2) ? 1 : v_qg);
  const int v_st = (v_d8 * 8) * VSTR + v_kqp * 4;
  // fragment read bases
  const int k_rd = n32 * KSTR + hi * 8;        // + kb*32*KSTR + ks*16
  const int v_rd = n32 * VSTR + hi * 8;        // + db*32*VSTR + kc*16

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto load_tile = [&](int tile) {
    const int left = max(n_keys - tile * KT, 0) * (D * 2);               // valid bytes from this tile on
    const int64_t toff = (int64_t)tile * (KT * D);
    __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc((void*)(Kb + toff), 0, left, 0x00020000);
    __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc((void*)(Vb + toff), 0, left, 0x00020000);
    if (do_k) {
#pragma unroll
      for (int i = 0; i < K_LD; ++i) {
        u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(kr, k_go[i], 0, 0);
        kreg[i] = make_uint4(x[0], x[1], x[2], x[3]);
      }
    }
    if (v_on) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(vr, v_go + i * (D * 2), 0, 0);
        vreg[i] = make_uint4(x[0], x[1], x[2], x[3]);
      }
    }
  };
  auto store_tile = [&](auto bufc) {
    constexpr int buf = decltype(bufc)::value;
    if (do_k) {
#pragma unroll
      for (int i = 0; i < K_LD; ++i) *(uint4*)(&sm.K[buf][k_st[i]]) = kreg[i];
    }
    if (v_on) {
      const uint32_t* r0 = (const uint32_t*)&vreg[0];
      const uint32_t* r1 = (const uint32_t*)&vreg[1];
      const uint32_t* r2 = (const uint32_t*)&vreg[2];
      const uint32_t* r3 = (const uint32_t*)&vreg[3];
#pragma unroll
      for (int p = 0; p < 4; ++p) {            // word p holds dims 2p (low half) and 2p+1 (high half)
        uint2 even, odd;
        even.x = (r0[p] & 0xffffu) | (r1[p] << 16);
        even.y = (r2[p] & 0xffffu) | (r3[p] << 16);
        odd.x = (r0[p] >> 16) | (r1[p] & 0xffff0000u);
        odd.y = (r2[p] >> 16) | (r3[p] & 0xffff0000u);
        *(uint2*)(&sm.Vt[buf][v_st + (2 * p) * VSTR]) = even;
        *(uint2*)(&sm.Vt[buf][v_st + (2 * p + 1) * VSTR]) = odd;
      }
    }
  };

  // ---- one tile: S^T = K Q^T, online softmax, O^T += V^T P^T ------------------------------------
  auto compute_tile = [&](auto bufc, int tile) {
    constexpr int buf = decltype(bufc)::value;
    const int base = tile * KT;
    if (base > wave_last_slot) return;         // wave-uniform: nothing this wavefront may see
    // K fragments are read a few steps ahead of the MFMAs that consume them, and the two 32-key
    // blocks alternate so that consecutive MFMAs never wait on each other's accumulator.
    f32x16 sacc[2][QB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) sacc[kb][qb] = negm[qb];
    {
      bf16x8 kf[NKS][2];
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kf[ks][kb] = *(const bf16x8*)(&sm.K[buf][k_rd + kb * 32 * KSTR + ks * 16]);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            sacc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks][kb], qf[qb][ks], sacc[kb][qb], 0, 0, 0);
      constexpr int AHEAD = 6;                      // fragments in flight
      __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
      for (int i = 0; i < 2 * NKS - AHEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, AHEAD * QB, 0);
    }
    uint4 pb[QB][4];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (base + KT - 1 > n_c + tw0 + qb * 32) {                     // wave-uniform: tile crosses the diagonal
        const int limit = n_c + min(tw0 + qb * 32 + n32, Tn - 1);    // last visible slot of this lane's query
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int slot = base + kb * 32 + (r >> 2) * 8 + hi * 4 + (r & 3);
            if (slot > limit) sacc[kb][qb][r] = -INFINITY;
          }
      }
      // exponentiate, pack to bf16 and sum (plain adds: v_dot2c shares the matrix pipe and queues behind
      // the other wavefront's MFMAs)
      float ps;
      auto exp_pack_sum = [&]() {
        float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          uint32_t w[8];
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            const float e0 = __builtin_amdgcn_exp2f(sacc[kb][qb][r]), e1 = __builtin_amdgcn_exp2f(sacc[kb][qb][r + 1]);
            w[r >> 1] = pack_bf16(e0, e1);
            ps0 += e0;
            ps1 += e1;
          }
          pb[qb][kb * 2 + 0] = make_uint4(w[0], w[1], w[2], w[3]);
          pb[qb][kb * 2 + 1] = make_uint4(w[4], w[5], w[6], w[7]);
        }
        ps = ps0 + ps1;
      };
      exp_pack_sum();
      // The running max moves only on the first tile and when some lane's sum over its 32 keys reaches
      // RESCALE_SUM = 2^30 (any probability that large, an overflow included, shows there): then take the
      // row max, raise the running max by it, scale sum and accumulator, refresh negm, correct this
      // tile's logits (formed against the old max) and redo its probabilities.
      if (fresh || __any(!(ps < RESCALE_SUM))) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][qb][r]);
        mx = max_across_halves(mx);
        const float delta = fresh ? mx : fmaxf(mx, 0.f);
        const float alpha = fresh ? 0.f : __builtin_amdgcn_exp2f(-delta);   // nothing accumulated yet when fresh
        m_run[qb] += delta;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) negm[qb][r] = -m_run[qb];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[kb][qb][r] -= delta;
        exp_pack_sum();
      }
      l_run[qb] += ps;
    }
    fresh = false;
    {
      bf16x8 vf[4][NDB];
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
#pragma unroll
        for (int db = 0; db < NDB; ++db) vf[kc][db] = *(const bf16x8*)(&sm.Vt[buf][v_rd + db * 32 * VSTR + kc * 16]);
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kc][db], *(const bf16x8*)&pb[qb][kc], oacc[db][qb], 0, 0, 0);
      constexpr int AHEAD = 6;
      __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 1);
#pragma unroll
      for (int i = 0; i < 4 * NDB - AHEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, QB, 1);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, AHEAD * QB, 1);
    }
  };

  auto step = [&](auto bufc, int tile) {
    constexpr int buf = decltype(bufc)::value;
    if (tile + 1 < n_tiles) load_tile(tile + 1);
    compute_tile(bufc, tile);
    if (tile + 1 < n_tiles) store_tile(IntC<buf ^ 1>());
    __syncthreads();
  };

  load_tile(0);
  store_tile(IntC<0>());
  __syncthreads();
  int tile = 0;
  for (; tile + 1 < n_tiles; tile += 2) {
    step(IntC<0>(), tile);
    step(IntC<1>(), tile + 1);
  }
  if (tile < n_tiles) step(IntC<0>(), tile);

  // ---- epilogue: O = O^T / l, lane holds 4 consecutive dims per (db, r/4) for its query -------------
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int t = tw0 + qb * 32 + n32;
    float l = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    if (t < Tn) {
      const float inv = 1.f / l;
      bf16_t* op = out + ((int64_t)t * h + j) * D;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          uint2 w;
          w.x = pack_bf16(oacc[db][qb][rq * 4 + 0] * inv, oacc[db][qb][rq * 4 + 1] * inv);
          w.y = pack_bf16(oacc[db][qb][rq * 4 + 2] * inv, oacc[db][qb][rq * 4 + 3] * inv);
          *(uint2*)(op + db * 32 + rq * 8 + hi * 4) = w;
        }
    }
  }
}

template <int D, int QB, int NW, int WPE>
static void attn_launch(const Dims& Dm, LaunchTimer tm, const void* q, const float2* tab, const void* Kx, const void* V, void* out, int T,
                        int n_c, float scale, hipStream_t st, const HeadLens& hl) {
  const int g = Dm.g;
  const int hpw = (NW == 8 && g % 8 == 0) ? 8 : (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
  const int wph = NW / hpw;
  const int TW = wph * 32 * QB;
  const int n_hgroups = Dm.h / hpw;
  const int n_ttiles = (T + TW - 1) / TW;
  const float c_log2 = scale * 1.4426950408889634f;
  const int spread = hl.ragged && Dm.tune.pp_spread != 0;
  const int n_wg = spread ? n_hgroups * ((n_ttiles + 7) / 8) * 8 : n_hgroups * n_ttiles;
  hipExtLaunchKernelGGL((attn_mfma_kernel<D, QB, NW, WPE>), dim3(n_wg), dim3(NW * 64), 0, st, tm.start, tm.stop,
                        0, (const bf16_t*)q, tab,
                     (const bf16_t*)Kx, (const bf16_t*)V, (bf16_t*)out, T, Dm.h, g, Dm.cap, n_c, c_log2, hpw,
                     n_hgroups, n_ttiles, hl, spread, longest_first(hl, Dm.h_kv));
}

// The direct-to-LDS kernel (attention_pp.hip) serves head dims 128 and 96 while byte offsets inside one head's
// cache fit 31 bits; everything else, and every shape when the context's switches ask for it, runs on the
// register-staged kernel above.
static bool pp_applies(const Dims& Dm) {
  return !Dm.tune.attn_regstaged && (Dm.d == 128 || Dm.d == 96) && (int64_t)Dm.cap * Dm.d * 2 < (1ll << 31);
}

// true when launch_attention_bf16 hands its LaunchTimer to the kernel's own dispatch
bool attention_bf16_attaches_timer(const Dims& Dm) { return Dm.d == 64 || Dm.d == 96 || Dm.d == 128; }

// the matrix-core kernels take un-rotated queries and rotate them themselves
bool attention_bf16_rotates_q(const Dims& Dm) { return Dm.rope; }

bool attention_bf16_fuses_select(const Dims& Dm, int n_cand) {
  return Dm.bf16 && Dm.tune.fuse_select && pp_applies(Dm) && attention_pp_fuses_select(Dm, n_cand);
}

void launch_attention_bf16(const Dims& Dm, const void* q, const void* Kx, const void* V, void* out, int T, int n_c,
                           float scale, hipStream_t st, const float2* q_rot_tab, LaunchTimer tm, const SelectArgs* sel,
                           const HeadLens* n_c_h, float* split_part, size_t split_floats) {
  const HeadLens hl = head_lens_or_common(n_c_h);
  if (pp_applies(Dm) && launch_attention_bf16_pp(Dm, tm, q, q_rot_tab, Kx, V, out, T, n_c, scale, st, sel, n_c_h, split_part, split_floats)) return;
#define LOCRET_CASE(DD)                                                                        \
  case DD:                                                                                     \
    attn_launch<DD, 1, 8, 2>(Dm, tm, q, q_rot_tab, Kx, V, out, T, n_c, scale, st, hl);           \
    break;
  switch (Dm.d) {
    LOCRET_CASE(64)
    LOCRET_CASE(96)
    LOCRET_CASE(128)
    default: launch_attention_simple(Dm, q, Kx, V, out, T, n_c, scale, st, n_c_h);
  }
#undef LOCRET_CASE
}

}  // namespace locret
