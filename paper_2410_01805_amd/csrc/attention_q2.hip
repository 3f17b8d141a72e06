// Chunk attention (Eq. 1) on the bf16 matrix cores of gfx950, head_dim 128, 64 queries per wavefront.
//
// The direct-to-LDS kernel of attention_dma.hip with four wavefronts per workgroup (one per SIMD) that
// each own TWO blocks of 32 queries: every K and V^T fragment read from LDS feeds two MFMAs instead of
// one, which halves the LDS traffic per flop (the other kernels spend one 1 KB fragment read per MFMA).
// The accumulators of two query blocks need the whole register file of a SIMD, so no second wavefront
// is there to fill the matrix pipe during the softmax; the wavefront overlaps it with its own MFMAs
// instead: a 64-key tile is processed as two halves of 32 keys, and the S block of the next half is
// issued slot by slot between the exp2 / pack / add of the current one (the two are independent).
//
//   iteration t:  wait own loads of tile t+1, barrier, start the loads of tile t+3
//                 [ S(t, keys 32..63) | softmax(t, keys 0..31) ]   PV(t, keys 0..31)
//                 [ S(t+1, keys 0..31) | softmax(t, keys 32..63) ] PV(t, keys 32..63)
//
// Ring of 4 stages, one tile and one barrier per iteration; invariant at the barrier of iteration t:
// tiles up to t+1 are in LDS (every wavefront waits for its own loads with s_waitcnt vmcnt(8): only the
// 8 loads of tile t+2 may still be in flight) and every wavefront has left iteration t-1, so the stage
// of tile t-1 is free for tile t+3.
//
// The running max is moved as in the other kernels (first tile, or a probability sum of a half tile
// reaching 2^30); the S block issued beside the softmax was formed against the old max and is corrected
// on that rare path.  V^T fragments are read from inline assembly with hand-counted lgkmcnt waits (see
// attention_pp.hip).  This file is compiled with -mllvm -amdgpu-mfma-vgpr-form: without it every MFMA
// writes AGPRs and each logit costs a copy before its exp2.
//
// Tile layout in LDS, swizzles and fragment addressing are those of attention_dma.hip.
#include <hip/hip_ext.h>

#include "attn_common.h"
#include "kernels.h"

namespace locret {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(3))) unsigned char* lds_u8_ptr;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int Q2_D = 128;
constexpr int Q2_TILE_B = KT * Q2_D * 2;       // 16 KB per operand tile
constexpr int Q2_STAGE_B = 2 * Q2_TILE_B;      // K then V
constexpr int Q2_NW = 4;
constexpr int Q2_KPRE = 4;                     // K fragments requested ahead of their MFMAs
constexpr int Q2_VPRE = 4;                     // V^T fragments in flight ahead of their MFMAs

#define LOCRET_TR_READ(dst, addr, off) \
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(off) : "memory")
#define LOCRET_LGKM_WAIT(a, b, n) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "i"(n))

__global__ __launch_bounds__(Q2_NW * 64, 1) void attn_q2_kernel(const bf16_t* __restrict__ q, const float2* __restrict__ tab, const bf16_t* __restrict__ Kx,
                                                             const bf16_t* __restrict__ V, bf16_t* __restrict__ out,
                                                             int Tn, int h, int g, int cap, int n_c, float c_log2,
                                                             int hpw, int n_hgroups, int n_ttiles) {
  constexpr int NW = Q2_NW;
  constexpr int D = Q2_D;
  constexpr int NKS = D / 16;
  constexpr int NDB = D / 32;
  __shared__ __attribute__((aligned(1024))) unsigned char ring[4 * Q2_STAGE_B];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31;
  const int hi = lane >> 5;

  const int bid = blockIdx.x;
  int hgroup, tt;
  if ((n_hgroups & 7) == 0) {                  // one KV head per XCD (workgroup ids go round the XCDs)
    const int g8 = n_hgroups >> 3;
    hgroup = (bid & 7) * g8 + (bid >> 3) % g8;
    tt = bid / n_hgroups;
  } else {
    hgroup = bid % n_hgroups;
    tt = bid / n_hgroups;
  }
  tt = n_ttiles - 1 - tt;                      // longest key ranges first
  const int wph = NW / hpw;                    // wavefronts per query head
  const int TW = wph * 64;
  const int t0 = tt * TW;
  const int j = hgroup * hpw + wave / wph;
  const int m = (hgroup * hpw) / g;
  const int tw0 = t0 + (wave % wph) * 64;
  const int t_last_wg = min(Tn, t0 + TW) - 1;
  const int n_keys = n_c + t_last_wg + 1;
  const int n_tiles = (n_keys + KT - 1) / KT;
  const int wave_last_slot = n_c + min(Tn - 1, tw0 + 63);
  int limit[2];                                // last visible slot of this lane's query, per query block

  auto scalar_ptr = [](const bf16_t* p) -> const bf16_t* {
    uint64_t a = (uint64_t)p;
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    uint32_t hi32 = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return (const bf16_t*)(((uint64_t)hi32 << 32) | lo);
  };
  const bf16_t* Kb = scalar_ptr(Kx + (int64_t)m * cap * D);
  const bf16_t* Vb = scalar_ptr(V + (int64_t)m * cap * D);

  bf16x8 qf[2][NKS];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int my_t = min(tw0 + qb * 32 + n32, Tn - 1);
    limit[qb] = n_c + my_t;
    const bf16_t* qp = q + ((int64_t)my_t * h + j) * D + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[qb][ks] = *(const bf16x8*)(qp + ks * 16);
    const float qscale = c_log2;                 // logits come out of the MFMA in log2 units
    if (tab != nullptr) {
      // un-rotated queries: rotate to position n_c + t here (pairs (i, i + D/2) sit in fragments ks
      // and ks + NKS/2 of the same lane), round to bf16 as the append kernel would have
      const float2* tp = tab + (int64_t)(n_c + my_t) * (D / 2) + hi * 8;
#pragma unroll
      for (int ks = 0; ks < NKS / 2; ++ks) {
        float lo[8], up[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float2 cs = tp[ks * 16 + e];
          const float a = (float)qf[qb][ks][e], b = (float)qf[qb][ks + NKS / 2][e];
          lo[e] = (a * cs.x - b * cs.y) * qscale;
          up[e] = (b * cs.x + a * cs.y) * qscale;
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
        for (int e = 0; e < 8; ++e) x[e] = (float)qf[qb][ks][e] * qscale;
        uint4 px = make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
        qf[qb][ks] = __builtin_bit_cast(bf16x8, px);
      }
    }
  }
  // the query fragments are only ever MFMA B operands: held in accumulation registers from here on
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) asm volatile("" : "+a"(qf[qb][ks]));
  f32x16 oacc[2][NDB];
  f32x16 negm[2];                              // -(running max), log2 units, in all 16 registers
  float m_run[2] = {0.f, 0.f}, l_run[2] = {0.f, 0.f};
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[qb][r] = 0.f;
  }
  // the output accumulators live in accumulation registers: only the PV MFMAs (inline asm below) touch them on
  // the common path; every other definition is followed by a pin so that the loop-carried value keeps that class
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int db = 0; db < NDB; ++db) asm volatile("" : "+a"(oacc[qb][db]));
  bool fresh = true;                           // wave-uniform: no tile half has set the max yet

  // ---- direct loads: instruction i of a tile covers rows 4i .. 4i+3; wavefront w issues instructions
  // ---- w + 4u of K and of V, so (i & 3) = w for all of them -------------------------------------------
  const int l_row = lane >> 4, l_pos = lane & 15;
  const int k_vo = wave * 1024 + l_row * 256 + ((l_pos ^ l_row ^ (wave << 2)) * 16);   // + u * 4096 (scalar offset)
  const int v_vo = wave * 1024 + l_row * 256 + ((l_pos ^ (l_row << 2)) * 16);
  auto issue = [&](int tile, int stage) __attribute__((always_inline)) {
    const int tile_u = __builtin_amdgcn_readfirstlane(tile);
    const int left = __builtin_amdgcn_readfirstlane(max(n_keys - tile_u * KT, 0) * (D * 2));   // 0 past the end
    __amdgpu_buffer_rsrc_t kr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Kb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
    __amdgpu_buffer_rsrc_t vr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Vb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
    unsigned char* sb = ring + stage * Q2_STAGE_B;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = wave + u * 4;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, (lds_ptr_t)(sb + i * 1024), 16, k_vo, u * 4096, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = wave + u * 4;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, (lds_ptr_t)(sb + Q2_TILE_B + i * 1024), 16, v_vo, u * 4096, 0, 0);
    }
  };

  // ---- fragment addresses (bytes inside a stage) ---------------------------------------------------
  const int kx = n32 & 15;
  const int k_base = n32 * 256 + ((kx >> 1) << 5) + ((hi ^ (kx & 1)) << 4);
  int k_rd[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) k_rd[ks] = k_base ^ (ks << 5);
  const int vs = lane & 15, vG = lane >> 4;
  const int v_base = Q2_TILE_B + (((vG >> 1) * 4 + (vs >> 2)) * 256) + ((vs >> 2) << 6) +
                     ((((vG & 1) << 1) + ((vs & 3) >> 1)) << 4) + ((vs & 1) << 3);
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(lds_u8_ptr)ring;
  uint32_t v_ad[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) v_ad[db] = ring_lds + (uint32_t)(v_base ^ (db << 6));

  // S of one half tile (32 keys) for both query blocks, nothing beside it (the very first half)
  auto s_half = [&](f32x16 (&s)[2], int sb_off, int half) __attribute__((always_inline)) {
    const unsigned char* sb = ring + sb_off + half * (32 * 256);
    bf16x8 kf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) kf[ks] = *(const bf16x8*)(sb + k_rd[ks]);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
        s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[qb][ks], ks == 0 ? negm[qb] : s[qb], 0, 0, 0);
  };

  // exp2, pack and sum of one half tile's logits, nothing beside it (the rare path)
  auto exp_pack_sum = [&](const f32x16 (&c)[2], uint4 (&pb)[2][2], float (&ps)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      uint32_t w[8];
      float p0 = 0.f, p1 = 0.f;
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float e0 = __builtin_amdgcn_exp2f(c[qb][r]), e1 = __builtin_amdgcn_exp2f(c[qb][r + 1]);
        w[r >> 1] = pack_bf16(e0, e1);
        p0 += e0;
        p1 += e1;
      }
      pb[qb][0] = make_uint4(w[0], w[1], w[2], w[3]);
      pb[qb][1] = make_uint4(w[4], w[5], w[6], w[7]);
      ps[qb] = p0 + p1;
    }
  };

  // One half step: S of the next half tile into nxt, slot by slot beside the softmax of cur (whose keys
  // are half `half` of tile `tile`); then the rare running-max move; then PV of cur's half.
  auto half_step = [&](int tile, int half, f32x16 (&cur)[2], f32x16 (&nxt)[2], int sb_cur, int sb_nxt, int half_nxt) __attribute__((always_inline)) {
    const int base = tile * KT + half * 32;
    if (tile * KT + KT - 1 > n_c + tw0) {      // wave-uniform: the tile crosses the diagonal
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int slot = base + (r >> 2) * 8 + hi * 4 + (r & 3);
          if (slot > limit[qb]) cur[qb][r] = -INFINITY;
        }
    }
    uint4 pb[2][2];
    float ps[2];
    {
      const unsigned char* sb = ring + sb_nxt + half_nxt * (32 * 256);
      bf16x8 kf[NKS];
#pragma unroll
      for (int ks = 0; ks < Q2_KPRE; ++ks) kf[ks] = *(const bf16x8*)(sb + k_rd[ks]);
      uint32_t w[2][8];
      float p[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
      uint32_t wp0 = 0, wp1 = 0;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        // slot ks: the two MFMAs of K fragment ks, the read of fragment ks + KPRE, and logits
        // 4 (ks % 4) .. + 3 of query block ks / 4.  The fragment and the logits pass through an empty asm
        // statement (ordered with the others), which keeps each slot's vector work inside the slot.
        const int qs = ks >> 2, r0 = (ks & 3) * 4;
        float c0 = cur[qs][r0], c1 = cur[qs][r0 + 1], c2 = cur[qs][r0 + 2], c3 = cur[qs][r0 + 3];
        asm volatile("" : "+v"(kf[ks]), "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3), "+v"(p[0][0]), "+v"(p[0][1]),
                          "+v"(p[1][0]), "+v"(p[1][1]), "+v"(wp0), "+v"(wp1));
        if (ks > 0) {
          w[(ks - 1) >> 2][((ks - 1) & 3) * 2] = wp0;
          w[(ks - 1) >> 2][((ks - 1) & 3) * 2 + 1] = wp1;
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
          nxt[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[qb][ks], ks == 0 ? negm[qb] : nxt[qb], 0, 0, 0);
        if (ks + Q2_KPRE < NKS) kf[ks + Q2_KPRE] = *(const bf16x8*)(sb + k_rd[ks + Q2_KPRE]);
        const float e0 = __builtin_amdgcn_exp2f(c0), e1 = __builtin_amdgcn_exp2f(c1);
        const float e2 = __builtin_amdgcn_exp2f(c2), e3 = __builtin_amdgcn_exp2f(c3);
        wp0 = pack_bf16(e0, e1);
        wp1 = pack_bf16(e2, e3);
        p[qs][0] += e0 + e2;
        p[qs][1] += e1 + e3;
        __builtin_amdgcn_sched_barrier(0);
      }
      asm volatile("" : "+v"(wp0), "+v"(wp1), "+v"(p[0][0]), "+v"(p[0][1]), "+v"(p[1][0]), "+v"(p[1][1]));
      w[1][6] = wp0;
      w[1][7] = wp1;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        pb[qb][0] = make_uint4(w[qb][0], w[qb][1], w[qb][2], w[qb][3]);
        pb[qb][1] = make_uint4(w[qb][4], w[qb][5], w[qb][6], w[qb][7]);
        ps[qb] = p[qb][0] + p[qb][1];
      }
    }
    if (fresh || __any(!(ps[0] < RESCALE_SUM) || !(ps[1] < RESCALE_SUM))) {   // rare: move the running max
      // the accumulators are re-defined here (an empty statement): what the rescale below needs of them is then
      // copied inside this block and not, hoisted, at the top of every iteration
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < NDB; ++db) asm volatile("" : "+a"(oacc[qb][db]));
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, cur[qb][r]);
        mx = max_across_halves(mx);
        const float delta = fresh ? mx : fmaxf(mx, 0.f);
        const float alpha = fresh ? 0.f : __builtin_amdgcn_exp2f(-delta);   // nothing accumulated yet when fresh
        m_run[qb] += delta;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db) asm volatile("" : "+a"(oacc[qb][db]));
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          negm[qb][r] = -m_run[qb];
          cur[qb][r] -= delta;
          nxt[qb][r] -= delta;                 // formed against the old max
        }
      }
      fresh = false;
      exp_pack_sum(cur, pb, ps);
    }
    l_run[0] += ps[0];
    l_run[1] += ps[1];
    // ---- PV of the half: V^T fragment f = kc * NDB + db (kc = 16-key chunk inside the half), two
    // ---- transposing 8-byte reads each, every fragment feeds both query blocks ----
    uint32_t va[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db) va[db] = v_ad[db] + (uint32_t)(sb_cur + half * (2 * 4096));
    s16x4 vlo[2 * NDB], vhi[2 * NDB];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < Q2_VPRE; ++f) {
      LOCRET_TR_READ(vlo[f], va[f % NDB], (f / NDB) * 4096);
      LOCRET_TR_READ(vhi[f], va[f % NDB], (f / NDB) * 4096 + 2048);
    }
#pragma unroll
    for (int f = 0; f < 2 * NDB; ++f) {
      constexpr int LASTF = 2 * NDB - 1;
      const int newest = f + Q2_VPRE - 1 < LASTF ? f + Q2_VPRE - 1 : LASTF;   // newest fragment already requested
      static_assert(Q2_VPRE <= 4, "lgkmcnt cases");
      switch (2 * (newest - f)) {              // reads issued after fragment f's: two per fragment
        case 6: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 6); break;
        case 4: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 4); break;
        case 2: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 2); break;
        default: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 0); break;
      }
      const s16x8 both = __builtin_shufflevector(vlo[f], vhi[f], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
      {
        const bf16x8 pfrag = *(const bf16x8*)&pb[qb][f / NDB];
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(oacc[qb][f % NDB]) : "v"(both), "v"(pfrag));
      }
      if (f + Q2_VPRE < 2 * NDB) {
        const int fn = f + Q2_VPRE;
        LOCRET_TR_READ(vlo[fn], va[fn % NDB], (fn / NDB) * 4096);
        LOCRET_TR_READ(vhi[fn], va[fn % NDB], (fn / NDB) * 4096 + 2048);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  auto top = [&](int t) __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");             // own loads of tile t+1 have landed
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    issue(t + 3, (t + 3) & 3);
  };

  // ---- ring ---------------------------------------------------------------------------------------
  // tiles this wavefront's queries can see (wave-uniform, <= n_tiles): later tiles only keep the barriers
  const int n_active = min(n_tiles, wave_last_slot / KT + 1);
  issue(0, 0);
  issue(1, 1);
  issue(2, 2);
  asm volatile("s_waitcnt vmcnt(8)" ::: "memory");               // own loads of tiles 0 and 1 have landed
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_barrier" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  f32x16 sA[2], sB[2];
  s_half(sA, 0, 0);                                              // S of tile 0, keys 0..31
  for (int t = 0; t < n_active; ++t) {
    top(t);
    const int sb_cur = (t & 3) * Q2_STAGE_B, sb_nx = ((t + 1) & 3) * Q2_STAGE_B;
    half_step(t, 0, sA, sB, sb_cur, sb_cur, 1);
    half_step(t, 1, sB, sA, sb_cur, sb_nx, 0);
  }
  for (int t = n_active; t < n_tiles; ++t) top(t);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // trailing empty loads

  // ---- epilogue ---------------------------------------------------------------------------------
  // the MFMAs that wrote the accumulators are inline assembly, whose results the compiler's hazard handling does
  // not track: leave the matrix pipe's write-back time before the first read
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7"
               : "+a"(oacc[0][0]), "+a"(oacc[0][1]), "+a"(oacc[0][2]), "+a"(oacc[0][3]), "+a"(oacc[1][0]), "+a"(oacc[1][1]),
                 "+a"(oacc[1][2]), "+a"(oacc[1][3]));
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int t = tw0 + qb * 32 + n32;
    const float l = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    if (t < Tn) {
      const float inv = 1.f / l;
      bf16_t* op = out + ((int64_t)t * h + j) * D;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          uint2 w;
          w.x = pack_bf16(oacc[qb][db][rq * 4 + 0] * inv, oacc[qb][db][rq * 4 + 1] * inv);
          w.y = pack_bf16(oacc[qb][db][rq * 4 + 2] * inv, oacc[qb][db][rq * 4 + 3] * inv);
          *(uint2*)(op + db * 32 + rq * 8 + hi * 4) = w;
        }
    }
  }
}

// `tab` non-null: q holds un-rotated queries and the kernel rotates them (table row n_c + t).
bool launch_attention_bf16_q2(const Dims& Dm, LaunchTimer tm, const void* q, const float2* tab, const void* Kx, const void* V, void* out,
                              int T, int n_c, float scale, hipStream_t st) {
  if (Dm.d != Q2_D) return false;
  if ((int64_t)Dm.cap * Dm.d * 2 >= (1ll << 31)) return false;   // 32-bit byte offsets inside one head
  constexpr int NW = Q2_NW;
  const int g = Dm.g;
  const int hpw = (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
  const int wph = NW / hpw;
  const int TW = wph * 64;
  const int n_hgroups = Dm.h / hpw;
  const int n_ttiles = (T + TW - 1) / TW;
  const float c_log2 = scale * 1.4426950408889634f;
  hipExtLaunchKernelGGL(attn_q2_kernel, dim3(n_hgroups * n_ttiles), dim3(NW * 64), 0, st, tm.start, tm.stop, 0,
                        (const bf16_t*)q, tab, (const bf16_t*)Kx, (const bf16_t*)V, (bf16_t*)out, T, Dm.h, g, Dm.cap, n_c,
                        c_log2, hpw, n_hgroups, n_ttiles);
  return true;
}

}  // namespace locret
